// GLM iteration on a sparse X held in CSR (rows) and CSC (columns) form.
//
// Both passes are the same deterministic segmented sum  out[s] = sum_{e in segment s} val[e] * vec[idx[e]]
// (rows: vec = w, out = margins; columns: vec = residuals, out = X^T r).  Work is split by
// ENTRIES, not by segments, so a few very long columns or rows cost no more than many short
// ones: a wave owns a chunk of 512 consecutive entries, loads them coalesced, multiplies, and
// reduces inside the chunk; segments that cross chunk borders are completed by a fix-up kernel
// that adds the per-chunk pieces in chunk order.  No floating-point atomics: every sum has an
// order fixed by the layout of the matrix alone.
//
// Inside a chunk: the segment starts that fall inside it are marked in LDS (integer counts, so
// that empty segments advance the segment index too); lane l then walks entries 8 l .. 8 l + 7
// in order.  A segment that starts and ends inside one lane is written directly.  The open
// pieces at lane borders are combined by a segmented scan across the lanes (fixed shuffle tree).
// Per chunk three things may remain: the piece of the segment that was already open at the chunk
// start (H), the piece of the segment still open at the chunk end (T), or, if no segment starts
// inside the chunk, the whole chunk as one piece (also T).
#include "glm_internal.h"
#include "glm_loss.h"
#include "sparse_internal.h"

#include <cmath>

namespace slaqglm {

constexpr int kSpU = 8;                    // entries per lane
constexpr int kSpChunk = 64 * kSpU;        // entries per wave
static_assert(kSpChunk == kSparseChunk, "chunk size is part of the workspace layout");
constexpr int kSpPad = kSpChunk + kSpChunk / 32;

__device__ __forceinline__ int pad32(int p) { return p + (p >> 5); }   // breaks the stride-8 bank pattern

// seg0[c] = last segment s < S whose start ptr[s] is <= c * chunk (the segment that holds the
// chunk's first entry); seg0[nch] = S - 1.
__global__ void seg_start_kernel(const long long *__restrict__ ptr, long long S, long long nch,
                                 int *__restrict__ seg0) {
    const long long c = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (c > nch) return;
    if (c == nch) { seg0[c] = (int)(S - 1); return; }
    const long long e = c * kSpChunk;
    long long lo = 0, hi = S;              // invariant: ptr[lo] <= e (ptr[0] = 0), answer in [lo, hi)
    while (hi - lo > 1) {
        const long long mid = (lo + hi) >> 1;
        if (ptr[mid] <= e) lo = mid; else hi = mid;
    }
    seg0[c] = (int)lo;
}

struct ChunkRec {                          // per-chunk leftovers, one array each (structure of arrays)
    int *closes; int *headless; int *slast; float *H; float *T;
};

__global__ __launch_bounds__(256) void seg_sum_kernel(
    const long long *__restrict__ ptr, const int *__restrict__ idx, const float *__restrict__ val,
    const float *__restrict__ vec, long long E, long long nch, const int *__restrict__ seg0,
    float *__restrict__ out, ChunkRec rec) {
    __shared__ float prod_s[4][kSpPad];
    __shared__ int flag_s[4][kSpPad];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const long long c = (long long)blockIdx.x * 4 + wave;
    const bool active = c < nch;           // inactive waves still reach the barriers
    float *prod = prod_s[wave];
    int *flag = flag_s[wave];
    const long long e0 = c * kSpChunk;
    const long long e1 = active ? ((e0 + kSpChunk < E) ? e0 + kSpChunk : E) : e0;

    for (int p = lane; p < kSpPad; p += 64) flag[p] = 0;
    int s_lo = 0;
    bool headless = false;
    if (active) {
#pragma unroll
        for (int u = 0; u < kSpU; ++u) {
            const long long e = e0 + u * 64 + lane;
            float p = 0.0f;
            if (e < e1) p = __builtin_nontemporal_load(val + e) * vec[__builtin_nontemporal_load(idx + e)];
            prod[pad32(u * 64 + lane)] = p;
        }
        s_lo = seg0[c];
        headless = ptr[s_lo] == e0;
    }
    __syncthreads();                       // flags are zero before anyone marks
    if (active) {
        const int s_up = seg0[c + 1];
        for (int s = s_lo + 1 + lane; s <= s_up; s += 64) {
            const long long pe = ptr[s];
            if (pe < e1) atomicAdd(&flag[pad32((int)(pe - e0))], 1);    // integer count: order-free
        }
    }
    __syncthreads();
    if (!active) return;

    // this lane's eight entries, and how many segment starts lie in them
    float pv[kSpU]; int fv[kSpU];
    int cnt = 0;
#pragma unroll
    for (int u = 0; u < kSpU; ++u) {
        pv[u] = prod[pad32(lane * kSpU + u)];
        fv[u] = flag[pad32(lane * kSpU + u)];
        cnt += fv[u];
    }
    int incl = cnt;                        // inclusive prefix of the counts over the lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
    }
    int cur = s_lo + (incl - cnt);         // segment open when this lane starts
    const int head_seg = cur;

    const int nvalid = (int)(e1 - e0);
    float acc = 0.0f, head = 0.0f;
    bool started = false, lane_closes = false;
#pragma unroll
    for (int u = 0; u < kSpU; ++u) {
        if (lane * kSpU + u < nvalid) {
            if (fv[u] > 0) {
                if (started) out[cur] = acc;                 // began and ended inside this lane
                else { head = acc; lane_closes = true; }
                cur += fv[u];
                acc = 0.0f;
                started = true;
            }
            acc += pv[u];
        }
    }
    // segmented inclusive scan of the open pieces: a lane that closes starts a new run
    float run = acc;
    int runf = lane_closes ? 1 : 0;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const float ov = __shfl_up(run, d, 64);
        const int of = __shfl_up(runf, d, 64);
        if (lane >= d) {
            if (!runf) run = ov + run;
            runf |= of;
        }
    }
    float cin = __shfl_up(run, 1, 64);
    int prevf = __shfl_up(runf, 1, 64);
    if (lane == 0) { cin = 0.0f; prevf = 0; }
    if (lane_closes) {
        const float tot = cin + head;
        if (prevf || headless) out[head_seg] = tot;          // the whole segment lies in this chunk
        else rec.H[c] = tot;                                 // it was already open at the chunk start
    }
    const int last_lane = (nvalid - 1) / kSpU;
    const int slast = __shfl(cur, last_lane, 64);
    if (lane == 63) {
        rec.closes[c] = runf;
        rec.headless[c] = headless ? 1 : 0;
        rec.slast[c] = slast;
        rec.T[c] = run;
    }
}

// Completes the segments that cross chunk borders.  The chunk in which such a segment starts
// (it closes a segment, or begins exactly at a segment start) owns it: its T, then the T of the
// following chunks that neither contain nor begin at a segment start, then the H of the chunk
// that closes it.  One lane per chunk settles the common case (the segment ends in the next
// chunk, or at its border); the owners of longer runs are then served one after another by the
// whole wave, 64 chunks per step, so a segment of millions of entries takes a few dozen steps.
__global__ __launch_bounds__(256) void seg_fixup_kernel(long long nch, ChunkRec rec, float *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    const long long c = blockIdx.x * 256LL + threadIdx.x;
    bool pending = false;
    if (c < nch && (rec.closes[c] || rec.headless[c])) {
        const float t = rec.T[c];
        const long long k = c + 1;
        if (k >= nch || rec.headless[k]) out[rec.slast[c]] = t;
        else if (rec.closes[k]) out[rec.slast[c]] = (float)((double)t + (double)rec.H[k]);
        else pending = true;
    }
    unsigned long long todo = __ballot(pending);
    while (todo) {
        const int src = __ffsll((long long)todo) - 1;
        todo &= todo - 1;
        const long long cs = c - lane + src;                  // the owner chunk being served
        double tot = (double)rec.T[cs];
        long long k0 = cs + 1;
        while (true) {
            const long long k = k0 + lane;
            const bool end = (k >= nch) || rec.headless[k];
            const bool cl = !end && rec.closes[k];
            const unsigned long long stop = __ballot(end || cl);
            const int fs = stop ? (__ffsll((long long)stop) - 1) : 64;
            double v = 0.0;
            if (lane < fs) v = (double)rec.T[k];
            else if (lane == fs && cl) v = (double)rec.H[k];
            for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
            tot += v;
            if (fs < 64) break;
            k0 += 64;
        }
        if (lane == src) out[rec.slast[cs]] = (float)tot;
    }
}

__global__ void fill_zero_kernel(float *__restrict__ p, long long n) {
    const long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

constexpr int kEpi = 8;                    // elements per thread of the epilogues

// For the fixed-point passes: the largest |v| of the block goes into *maxslot (bit patterns of
// non-negative floats order as unsigned integers; the maximum does not depend on the order), and
// block 0 clears *zeroslot, which the next kernel but one accumulates into.  Both may be null.
__device__ __forceinline__ void block_absmax(float v, unsigned *__restrict__ maxslot, unsigned *__restrict__ zeroslot) {
    __shared__ unsigned redm[4];
    if (maxslot) {
        unsigned m = __float_as_uint(v) & 0x7FFFFFFFu;
        for (int o = 32; o >= 1; o >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, o, 64));
        if ((threadIdx.x & 63) == 0) redm[threadIdx.x >> 6] = m;
        __syncthreads();
        if (threadIdx.x == 0) atomicMax(maxslot, max(max(redm[0], redm[1]), max(redm[2], redm[3])));
    }
    if (zeroslot && blockIdx.x == 0 && threadIdx.x == 0) *zeroslot = 0u;
}

// Sum over the 256 threads of a block in a fixed order: a butterfly inside each wave, then the
// four waves in order.  Valid in thread 0.
template <typename T>
__device__ __forceinline__ T block_sum_256(T v, T *red4) {
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    if ((threadIdx.x & 63) == 0) red4[threadIdx.x >> 6] = v;
    __syncthreads();
    return ((red4[0] + red4[1]) + red4[2]) + red4[3];
}

// Rows: margins -> loss and residual; per-block loss sums in a fixed tree.
__global__ __launch_bounds__(256) void sparse_row_epilogue(const float *__restrict__ z, const float *__restrict__ y,
                                                           long long N, int loss, float *__restrict__ r,
                                                           float *__restrict__ lossP, unsigned *__restrict__ maxslot,
                                                           unsigned *__restrict__ zeroslot) {
    __shared__ float red[4];
    // kEpi elements per thread, 256 apart: blocks of one element per thread are so short that
    // the kernel runs at the rate blocks can be started
    float l = 0.0f, rmag = 0.0f;
#pragma unroll
    for (int q = 0; q < kEpi; ++q) {
        const long long i = ((long long)blockIdx.x * kEpi + q) * 256 + threadIdx.x;
        if (i < N) {
            float lq, rr;
            loss_residual(loss, z[i], y[i], lq, rr);
            r[i] = rr;
            l += lq;
            rmag = __builtin_fmaxf(rmag, __builtin_fabsf(rr));
        }
    }
    block_absmax(rmag, maxslot, zeroslot);
    const float tot = block_sum_256(l, red);
    if (threadIdx.x == 0) lossP[blockIdx.x] = tot;
}

// Columns: X^T r -> gradient, update; per-block sums of w^2 (entering iterate) in a fixed tree.
__global__ __launch_bounds__(256) void sparse_col_epilogue(const float *__restrict__ gs, long long D, double invN,
                                                           float lambda, double step, float *__restrict__ w,
                                                           float *__restrict__ grad, double *__restrict__ wwP,
                                                           unsigned *__restrict__ maxslot,
                                                           unsigned *__restrict__ zeroslot) {
    __shared__ double red[4];
    double ww = 0.0;
    float wmag = 0.0f;
#pragma unroll
    for (int q = 0; q < kEpi; ++q) {
        const long long j = ((long long)blockIdx.x * kEpi + q) * 256 + threadIdx.x;
        if (j < D) {
            const float wj = w[j];
            const double g = (double)gs[j] * invN + (double)lambda * (double)wj;
            grad[j] = (float)g;
            ww += (double)wj * (double)wj;
            float wnew = wj;
            if (step != 0.0) { wnew = (float)((double)wj - step * g); w[j] = wnew; }
            wmag = __builtin_fmaxf(wmag, __builtin_fabsf(wnew));
        }
    }
    block_absmax(wmag, maxslot, zeroslot);
    const double tot = block_sum_256(ww, red);
    if (threadIdx.x == 0) wwP[blockIdx.x] = tot;
}

// loss_out = (sum lossP) / N + lambda / 2 * (sum wwP); thread t adds a contiguous run, then a fixed tree.
__global__ __launch_bounds__(1024) void sparse_loss_kernel(const float *__restrict__ lossP, long long nR,
                                                           const double *__restrict__ wwP, long long nC,
                                                           double invN, float lambda, float *__restrict__ loss_out) {
    __shared__ double redL[1024];
    __shared__ double redW[1024];
    const int t = threadIdx.x;
    double a = 0.0, b = 0.0;
    for (long long i = nR * t / 1024; i < nR * (t + 1) / 1024; ++i) a += (double)lossP[i];
    for (long long i = nC * t / 1024; i < nC * (t + 1) / 1024; ++i) b += wwP[i];
    redL[t] = a; redW[t] = b;
    __syncthreads();
    for (int s = 512; s >= 1; s >>= 1) {
        if (t < s) { redL[t] += redL[t + s]; redW[t] += redW[t + s]; }
        __syncthreads();
    }
    if (t == 0) *loss_out = (float)(redL[0] * invN + 0.5 * (double)lambda * redW[0]);
}

// Step of iteration k of this call under the job's schedule (host side, fp64).
static double sparse_step(const SparseArgs &a, int k) {
    const double eta = (double)a.step;
    return a.sched == GLM_STEP_INV_SQRT ? eta / std::sqrt((double)(a.k0 + k + 1)) : eta;
}

static hipError_t seg_pass(const long long *ptr, const int *idx, const float *val, const float *vec,
                           long long S, long long E, long long nch, int *seg0, float *out, ChunkRec rec,
                           hipStream_t st) {
    if (nch == 0) return hipSuccess;
    hipLaunchKernelGGL(seg_sum_kernel, dim3((unsigned)((nch + 3) / 4)), dim3(256), 0, st, ptr, idx, val, vec, E,
                       nch, seg0, out, rec);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(seg_fixup_kernel, dim3((unsigned)((nch + 255) / 256)), dim3(256), 0, st, nch, rec, out);
    (void)S;
    return hipGetLastError();
}

hipError_t launch_sparse_setup(const SparseArgs &a, hipStream_t st) {
    if (a.nch == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((a.nch + 1 + 255) / 256);
    hipLaunchKernelGGL(seg_start_kernel, dim3(blocks), dim3(256), 0, st, a.row_ptr, a.N, a.nch, a.seg0R);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(seg_start_kernel, dim3(blocks), dim3(256), 0, st, a.col_ptr, a.D, a.nch, a.seg0C);
    return hipGetLastError();
}

hipError_t launch_sparse_iteration(const SparseArgs &a, int k, hipEvent_t *ev, hipStream_t st) {
    hipError_t e;
    ChunkRec rec{a.closes, a.headless, a.slast, a.H, a.T};
    // z [N] and the column sums [D] are one allocation: clear both at once
    const long long nz = a.N + a.D;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, st, a.z, nz);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[0], st)) != hipSuccess) return e;
    if ((e = seg_pass(a.row_ptr, a.col_idx, a.row_val, a.w, a.N, a.nnz, a.nch, a.seg0R, a.z, rec, st)) != hipSuccess)
        return e;
    const unsigned nbR = (unsigned)((a.N + 256 * kEpi - 1) / (256 * kEpi)), nbC = (unsigned)((a.D + 256 * kEpi - 1) / (256 * kEpi));
    hipLaunchKernelGGL(sparse_row_epilogue, dim3(nbR), dim3(256), 0, st, a.z, a.y, a.N, a.loss, a.r, a.lossP, nullptr, nullptr);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = seg_pass(a.col_ptr, a.row_idx, a.col_val, a.r, a.D, a.nnz, a.nch, a.seg0C, a.gs, rec, st)) != hipSuccess)
        return e;
    if (ev && (e = hipEventRecord(ev[1], st)) != hipSuccess) return e;
    hipLaunchKernelGGL(sparse_col_epilogue, dim3(nbC), dim3(256), 0, st, a.gs, a.D, 1.0 / (double)a.N, a.lambda,
                       sparse_step(a, k), a.w, a.grad, a.wwP, nullptr, nullptr);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(sparse_loss_kernel, dim3(1), dim3(1024), 0, st, a.lossP, (long long)nbR, a.wwP,
                       (long long)nbC, 1.0 / (double)a.N, a.lambda, a.loss_out + k);
    return hipGetLastError();
}


// ---- Row-panelled column layout ------------------------------------------------------------

int sparse_panel_count(long long N, long long D) {
    if (N <= kSparsePanelRows + kSparsePanelRows / 2) return 1;
    long long P = (N + kSparsePanelRows - 1) / kSparsePanelRows;
    if (P > kSparseMaxPanels) P = kSparseMaxPanels;
    while (P > 1 && P * D >= (1LL << 31) - 8) --P;
    return (int)P;
}

// Are the rows of every column in ascending order?  One thread per pair of neighbouring entries;
// a descent is harmless only where the second entry starts a column (binary search, rare).
__global__ __launch_bounds__(256) void csc_sorted_kernel(const long long *__restrict__ col_ptr,
                                                         const int *__restrict__ row_idx, long long D,
                                                         long long nnz, int *__restrict__ flag) {
    const long long e = blockIdx.x * 256LL + threadIdx.x;
    if (e + 1 >= nnz) return;
    if (row_idx[e] <= row_idx[e + 1]) return;
    long long lo = 0, hi = D;                          // smallest c with col_ptr[c] >= e + 1 (col_ptr[D] = nnz)
    while (lo < hi) {
        const long long mid = (lo + hi) >> 1;
        if (col_ptr[mid] < e + 1) lo = mid + 1; else hi = mid;
    }
    if (col_ptr[lo] != e + 1) atomicOr(flag, 1);
}

// pp[p * D + col] = first entry of column col whose row is >= p R (p = 0 .. P)
__global__ void panel_bounds_kernel(const long long *__restrict__ col_ptr, const int *__restrict__ row_idx,
                                    long long D, int P, long long R, long long *__restrict__ pp) {
    const long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (t >= (long long)(P + 1) * D) return;
    const long long p = t / D, col = t - p * D;
    long long lo = col_ptr[col], hi = col_ptr[col + 1];
    const long long bound = p * R;
    while (lo < hi) {                                  // first entry with row >= bound
        const long long mid = (lo + hi) >> 1;
        if ((long long)row_idx[mid] < bound) lo = mid + 1; else hi = mid;
    }
    pp[t] = lo;
}

// Exclusive prefix sum of the segment lengths len[s] = pp[s + D] - pp[s], s = p D + col, in
// three steps: per block of 4096, the block totals (one thread; at most a few hundred thousand),
// and the final add.
__global__ __launch_bounds__(256) void panel_scan_block_kernel(const long long *__restrict__ pp, long long D,
                                                               long long S2, long long *__restrict__ ptr2,
                                                               long long *__restrict__ bsum) {
    __shared__ long long tot[256];
    const long long base = (long long)blockIdx.x * kScanBlock + threadIdx.x * 16LL;
    long long v[16], run = 0;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const long long s = base + q;
        v[q] = run;
        run += s < S2 ? pp[s + D] - pp[s] : 0;
    }
    tot[threadIdx.x] = run;
    __syncthreads();
    if (threadIdx.x == 0) {
        long long acc = 0;
        for (int t = 0; t < 256; ++t) { const long long x = tot[t]; tot[t] = acc; acc += x; }
        bsum[blockIdx.x] = acc;
    }
    __syncthreads();
    const long long off = tot[threadIdx.x];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const long long s = base + q;
        if (s < S2) ptr2[s] = v[q] + off;
    }
}

__global__ void panel_scan_tops_kernel(long long nb, long long *__restrict__ bsum) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    long long acc = 0;
    for (long long b = 0; b < nb; ++b) { const long long x = bsum[b]; bsum[b] = acc; acc += x; }
    bsum[nb] = acc;
}

__global__ __launch_bounds__(256) void panel_scan_add_kernel(long long S2, const long long *__restrict__ bsum,
                                                             long long nb, long long *__restrict__ ptr2) {
    const long long s = blockIdx.x * 256LL + threadIdx.x;
    if (s < S2) ptr2[s] += bsum[s / kScanBlock];
    if (s == S2) ptr2[S2] = bsum[nb];
}

// One wave per (panel, column) segment: copy its entries to their place in the panelled layout.
__global__ __launch_bounds__(256) void panel_copy_kernel(const long long *__restrict__ pp,
                                                         const long long *__restrict__ ptr2, long long S2,
                                                         long long D, const int *__restrict__ row_idx,
                                                         const float *__restrict__ col_val,
                                                         int *__restrict__ idx2, float *__restrict__ val2) {
    const int lane = threadIdx.x & 63;
    const long long s = blockIdx.x * 4LL + (threadIdx.x >> 6);
    if (s >= S2) return;
    const long long src = pp[s], n = pp[s + D] - src, dst = ptr2[s];
    for (long long i = lane; i < n; i += 64) {
        idx2[dst + i] = row_idx[src + i];
        val2[dst + i] = col_val[src + i];
    }
}

// Columns: sum of the P per-panel sums in panel order, then gradient, update, |w|^2 partials.
__global__ __launch_bounds__(256) void sparse_col_epilogue_panels(const float *__restrict__ gs2, int P, long long D,
                                                                  double invN, float lambda, double step,
                                                                  float *__restrict__ w, float *__restrict__ grad,
                                                                  double *__restrict__ wwP,
                                                                  unsigned *__restrict__ maxslot,
                                                                  unsigned *__restrict__ zeroslot) {
    __shared__ double red[4];
    double ww = 0.0;
    float wmag = 0.0f;
#pragma unroll
    for (int q = 0; q < kEpi; ++q) {
        const long long j = ((long long)blockIdx.x * kEpi + q) * 256 + threadIdx.x;
        if (j < D) {
            double s = 0.0;
            for (int p = 0; p < P; ++p) s += (double)gs2[(size_t)p * D + j];
            const float wj = w[j];
            const double g = s * invN + (double)lambda * (double)wj;
            grad[j] = (float)g;
            ww += (double)wj * (double)wj;
            float wnew = wj;
            if (step != 0.0) { wnew = (float)((double)wj - step * g); w[j] = wnew; }
            wmag = __builtin_fmaxf(wmag, __builtin_fabsf(wnew));
        }
    }
    block_absmax(wmag, maxslot, zeroslot);
    const double tot = block_sum_256(ww, red);
    if (threadIdx.x == 0) wwP[blockIdx.x] = tot;
}

hipError_t launch_sparse_sorted_check(const SparseArgs &a, const SparsePanels &pn, hipStream_t st) {
    hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(64), 0, st, reinterpret_cast<float *>(pn.flag), 1LL);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(csc_sorted_kernel, dim3((unsigned)((a.nnz + 255) / 256)), dim3(256), 0, st, a.col_ptr, a.row_idx,
                       a.D, a.nnz, pn.flag);
    return hipGetLastError();
}

hipError_t launch_sparse_panel_build(const SparseArgs &a, const SparsePanels &pn, hipStream_t st) {
    hipError_t e;
    const long long S2 = (long long)pn.P * a.D;
    const long long nbounds = (long long)(pn.P + 1) * a.D;
    hipLaunchKernelGGL(panel_bounds_kernel, dim3((unsigned)((nbounds + 255) / 256)), dim3(256), 0, st, a.col_ptr,
                       a.row_idx, a.D, pn.P, pn.R, pn.pp);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const long long nb = (S2 + kScanBlock - 1) / kScanBlock;
    hipLaunchKernelGGL(panel_scan_block_kernel, dim3((unsigned)nb), dim3(256), 0, st, pn.pp, a.D, S2, pn.ptr2, pn.bsum);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(panel_scan_tops_kernel, dim3(1), dim3(64), 0, st, nb, pn.bsum);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(panel_scan_add_kernel, dim3((unsigned)((S2 + 1 + 255) / 256)), dim3(256), 0, st, S2, pn.bsum, nb,
                       pn.ptr2);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(panel_copy_kernel, dim3((unsigned)((S2 + 3) / 4)), dim3(256), 0, st, pn.pp, pn.ptr2, S2, a.D,
                       a.row_idx, a.col_val, pn.idx2, pn.val2);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (a.nch == 0) return hipSuccess;
    hipLaunchKernelGGL(seg_start_kernel, dim3((unsigned)((a.nch + 1 + 255) / 256)), dim3(256), 0, st, pn.ptr2, S2, a.nch,
                       pn.seg0);
    return hipGetLastError();
}

hipError_t launch_sparse_iteration_panels(const SparseArgs &a, const SparsePanels &pn, int k, hipEvent_t *ev,
                                          hipStream_t st) {
    if (pn.P <= 1) return launch_sparse_iteration(a, k, ev, st);
    hipError_t e;
    ChunkRec rec{a.closes, a.headless, a.slast, a.H, a.T};
    const long long S2 = (long long)pn.P * a.D;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((a.N + 255) / 256)), dim3(256), 0, st, a.z, a.N);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((S2 + 255) / 256)), dim3(256), 0, st, pn.gs2, S2);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[0], st)) != hipSuccess) return e;
    if ((e = seg_pass(a.row_ptr, a.col_idx, a.row_val, a.w, a.N, a.nnz, a.nch, a.seg0R, a.z, rec, st)) != hipSuccess)
        return e;
    const unsigned nbR = (unsigned)((a.N + 256 * kEpi - 1) / (256 * kEpi)), nbC = (unsigned)((a.D + 256 * kEpi - 1) / (256 * kEpi));
    hipLaunchKernelGGL(sparse_row_epilogue, dim3(nbR), dim3(256), 0, st, a.z, a.y, a.N, a.loss, a.r, a.lossP, nullptr, nullptr);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = seg_pass(pn.ptr2, pn.idx2, pn.val2, a.r, S2, a.nnz, a.nch, pn.seg0, pn.gs2, rec, st)) != hipSuccess)
        return e;
    if (ev && (e = hipEventRecord(ev[1], st)) != hipSuccess) return e;
    hipLaunchKernelGGL(sparse_col_epilogue_panels, dim3(nbC), dim3(256), 0, st, pn.gs2, pn.P, a.D, 1.0 / (double)a.N,
                       a.lambda, sparse_step(a, k), a.w, a.grad, a.wwP, nullptr, nullptr);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(sparse_loss_kernel, dim3(1), dim3(1024), 0, st, a.lossP, (long long)nbR, a.wwP,
                       (long long)nbC, 1.0 / (double)a.N, a.lambda, a.loss_out + k);
    return hipGetLastError();
}

// One iteration with each product on the path chosen for it: fixed-point scatter (fx), the
// row-panelled column layout (pn, column pass only) or the plain segmented sums.
hipError_t launch_sparse_iteration_any(const SparseArgs &a, const SparsePanels &pn, const SparseFx &fx, int k,
                                       hipEvent_t *ev, hipStream_t st) {
    if (!fx.row.on && !fx.col.on) return launch_sparse_iteration_panels(a, pn, k, ev, st);
    hipError_t e;
    ChunkRec rec{a.closes, a.headless, a.slast, a.H, a.T};
    const bool panels = !fx.col.on && pn.P > 1;
    const long long S2 = (long long)pn.P * a.D;
    // the segmented sums add into their outputs: clear those
    if (!fx.row.on) {
        hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((a.N + 255) / 256)), dim3(256), 0, st, a.z, a.N);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (!fx.col.on) {
        float *dst = panels ? pn.gs2 : a.gs;
        const long long n = panels ? S2 : a.D;
        hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, dst, n);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (ev && (e = hipEventRecord(ev[0], st)) != hipSuccess) return e;
    if (fx.row.on) e = launch_sparse_fx_pass(fx, true, a.w, a.D, a.nnz, a.z, st);
    else e = seg_pass(a.row_ptr, a.col_idx, a.row_val, a.w, a.N, a.nnz, a.nch, a.seg0R, a.z, rec, st);
    if (e != hipSuccess) return e;
    const unsigned nbR = (unsigned)((a.N + 256 * kEpi - 1) / (256 * kEpi)), nbC = (unsigned)((a.D + 256 * kEpi - 1) / (256 * kEpi));
    // max |r| feeds the column pass's scale; max |w| is cleared here and refilled by the column epilogue
    hipLaunchKernelGGL(sparse_row_epilogue, dim3(nbR), dim3(256), 0, st, a.z, a.y, a.N, a.loss, a.r, a.lossP,
                       fx.col.on ? fx.slots + kFxSlotMaxR : nullptr, fx.row.on ? fx.slots + kFxSlotMaxW : nullptr);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (fx.col.on) e = launch_sparse_fx_pass(fx, false, a.r, a.N, a.nnz, a.gs, st);
    else if (panels) e = seg_pass(pn.ptr2, pn.idx2, pn.val2, a.r, S2, a.nnz, a.nch, pn.seg0, pn.gs2, rec, st);
    else e = seg_pass(a.col_ptr, a.row_idx, a.col_val, a.r, a.D, a.nnz, a.nch, a.seg0C, a.gs, rec, st);
    if (e != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[1], st)) != hipSuccess) return e;
    unsigned *mw = fx.row.on ? fx.slots + kFxSlotMaxW : nullptr, *zr = fx.col.on ? fx.slots + kFxSlotMaxR : nullptr;
    if (panels)
        hipLaunchKernelGGL(sparse_col_epilogue_panels, dim3(nbC), dim3(256), 0, st, pn.gs2, pn.P, a.D, 1.0 / (double)a.N,
                           a.lambda, sparse_step(a, k), a.w, a.grad, a.wwP, mw, zr);
    else
        hipLaunchKernelGGL(sparse_col_epilogue, dim3(nbC), dim3(256), 0, st, a.gs, a.D, 1.0 / (double)a.N, a.lambda,
                           sparse_step(a, k), a.w, a.grad, a.wwP, mw, zr);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(sparse_loss_kernel, dim3(1), dim3(1024), 0, st, a.lossP, (long long)nbR, a.wwP,
                       (long long)nbC, 1.0 / (double)a.N, a.lambda, a.loss_out + k);
    return hipGetLastError();
}

}  // namespace slaqglm
