// Sparse products by scatter into LDS with fixed-point sums.
//
// The segmented sums of glm_sparse.hip gather one value of the other vector per stored entry; with
// vectors of millions of elements every gather of a wave touches 64 different cache lines and
// the pass runs at the rate of the cache, not of memory.  Here the roles are turned round.  The
// outputs (rows of z = X w, or columns of s = X^T r) are cut into panels of 16384; the entries of
// a panel are stored together, ordered by the index of the OTHER dimension, so that
//   - the value gathered from the other vector moves monotonically through memory while the
//     panel streams by (a wave's 64 gathers fall into one or two cache lines), and
//   - the 16384 sums of the panel live in LDS (128 KB) and every product is added to its sum
//     there.
// Adding in LDS means atomics, and the order of floating-point atomics is not fixed.  So the sums
// are integers: a product p becomes round(p * 2^e) as a 64-bit integer, with e chosen from the
// largest magnitudes present so that no sum can overflow (|sum| 2^e < 2^62).  Integer addition
// is associative: whatever the order, the sum is the same, and reruns are bit-identical.  The
// resolution is 2^-(62 - log2 longest run) of the largest possible product: far finer than the
// 2^-24 of an fp32 product.
//
// Layout of a pass (built once per matrix, in the workspace): entries sorted by (panel of the
// output index, position in the source layout).  For the row pass the source is the caller's
// column layout (CSC: within a panel, columns ascend), for the column pass the row layout (CSR).
// Per entry 8 bytes: one word with the output index inside its panel (14 bits) and the index into
// the gathered vector relative to the start of its window of 2^18 elements (18 bits), and the value
// (fp32).  Because the gathered index ascends along the source, a window is a contiguous piece of
// the source, and the entries of one panel and one window form a contiguous run of the layout;
// every run is padded with zero entries to a multiple of 4096, so that each group of 4096 entries
// (what a block loads in one step) lies in one panel and one window, whose first index is kept
// per group.  The padded entry stream of all panels is cut into equal
// spans, one per block (popular columns make some panels hundreds of times larger than others, so
// work is shared by entries, not by panels): a block walks the panels its span touches and writes
// 16384 partial sums for each; a small kernel adds the slices of a panel and converts to fp32.
#include "sparse_internal.h"

#include <cmath>

namespace slaqglm {

namespace {

constexpr int kFxTile = 2048;            // entries per tile of the split (one wave, 32 steps of 64)
constexpr int kFxThreads = 1024;
constexpr int kFxUnroll = 1;             // groups of four entries per lane and round (1, 2, 3, 4 measured: 0.725, 0.740, 0.731, 0.726 ms)

// ------------------------------------------------------------------ building the layout

// The source is cut into tiles of at most kFxTile entries, none of which crosses the start of a
// window: wsrc[w] = first source entry whose owner (the gathered index) is >= w 2^18, tfirst[w] =
// first tile of window w.  One thread; W <= kFxMaxWindows.
__global__ void fx_tiles_kernel(const long long *__restrict__ ptr, long long M, long long nnz, int W,
                                long long *__restrict__ wsrc, long long *__restrict__ tfirst) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    long long prev = 0, tiles = 0;
    for (int w = 0; w <= W; ++w) {
        const long long m = (long long)w << kFxWindowBits;
        long long e = w == 0 ? 0 : w == W ? nnz : ptr[m < M ? m : M];
        e = e < prev ? prev : e > nnz ? nnz : e;       // whatever the pointer array holds
        wsrc[w] = e;
        if (w > 0) tiles += (e - prev + kFxTile - 1) / kFxTile;
        tfirst[w] = w == 0 ? 0 : tiles;
        prev = e;
    }
}

// The window of a tile and its source entries [e0, e1); tiles past the last window's are empty.
__device__ __forceinline__ int fx_tile_range(const long long *__restrict__ wsrc, const long long *__restrict__ tfirst,
                                             int W, long long tile, long long *e0, long long *e1) {
    int w = 0;
    for (int i = 1; i < W; ++i) w = tfirst[i] <= tile ? i : w;
    const long long b = wsrc[w] + (tile - tfirst[w]) * kFxTile, end = wsrc[w + 1];
    *e0 = b < end ? b : end;
    *e1 = b + kFxTile < end ? b + kFxTile : end;
    if (tile >= tfirst[W]) *e1 = *e0;
    return w;
}

// cnt[key * ntiles + tile] = entries of the tile whose output index lies in panel `key`
__global__ __launch_bounds__(256) void fx_hist_kernel(const int *__restrict__ idx, long long ntiles, int P, int W,
                                                      const long long *__restrict__ wsrc,
                                                      const long long *__restrict__ tfirst,
                                                      long long *__restrict__ cnt) {
    __shared__ int hist[4][kFxMaxPanels];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int i = lane; i < kFxMaxPanels; i += 64) hist[wave][i] = 0;
    __syncthreads();
    const long long tile = blockIdx.x * 4LL + wave;
    if (tile < ntiles) {
        long long e0, e1;
        fx_tile_range(wsrc, tfirst, W, tile, &e0, &e1);
        for (long long e = e0 + lane; e < e1; e += 64) {
            const unsigned key = min((unsigned)idx[e] >> kFxPanelBits, (unsigned)(P - 1));
            atomicAdd(&hist[wave][key], 1);
        }
    }
    __syncthreads();
    if (tile < ntiles)
        for (int k = lane; k < P; k += 64) cnt[(long long)k * ntiles + tile] = hist[wave][k];
}

// exclusive prefix sum of a[0 .. n), total to a[n]: blocks of 4096, block totals by one thread, add
__global__ __launch_bounds__(256) void fx_scan_block_kernel(long long *__restrict__ a, long long n,
                                                            long long *__restrict__ bsum) {
    __shared__ long long tot[256];
    const long long base = (long long)blockIdx.x * kScanBlock + threadIdx.x * 16LL;
    long long v[16], run = 0;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const long long s = base + q;
        v[q] = run;
        run += s < n ? a[s] : 0;
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
        if (s < n) a[s] = v[q] + off;
    }
}

__global__ void fx_scan_tops_kernel(long long nb, long long *__restrict__ bsum) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    long long acc = 0;
    for (long long b = 0; b < nb; ++b) { const long long x = bsum[b]; bsum[b] = acc; acc += x; }
    bsum[nb] = acc;
}

__global__ __launch_bounds__(256) void fx_scan_add_kernel(long long n, const long long *__restrict__ bsum, long long nb,
                                                          long long *__restrict__ a) {
    const long long s = blockIdx.x * 256LL + threadIdx.x;
    if (s < n) a[s] += bsum[s / kScanBlock];
    if (s == n) a[n] = bsum[nb];
}

// One thread (P W <= 16384 runs): run (p, w) holds the entries of panel p whose source lies in window
// w; after the prefix sum cnt[p * ntiles + tfirst[w]] is its exact start.  rstart = its start in the
// padded layout (every run is filled up to a multiple of kFxRun), rlen = its entries, shift = how
// far they move up, pstart[p] = start of panel p's first run.
__global__ void fx_pstart_kernel(const long long *__restrict__ cnt, long long ntiles, int P, int W,
                                 const long long *__restrict__ tfirst, long long *__restrict__ pstart,
                                 long long *__restrict__ shift, long long *__restrict__ rstart,
                                 long long *__restrict__ rlen) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    long long at = 0;
    for (int p = 0; p < P; ++p) {
        pstart[p] = at;
        for (int w = 0; w < W; ++w) {
            const long long s = cnt[(long long)p * ntiles + tfirst[w]];
            const long long len = cnt[(long long)p * ntiles + tfirst[w + 1]] - s;
            rstart[p * W + w] = at;
            rlen[p * W + w] = len;
            shift[p * W + w] = at - s;
            at += (len + kFxRun - 1) / kFxRun * kFxRun;
        }
    }
    pstart[P] = at;
}

// One block per run: the zero entries that fill it up, and the window start of each of its groups.
__global__ __launch_bounds__(256) void fx_pad_kernel(int W, long long cap, const long long *__restrict__ rstart,
                                                     const long long *__restrict__ rlen, unsigned *__restrict__ ent,
                                                     float *__restrict__ val, int *__restrict__ tbase) {
    const int w = (int)(blockIdx.x % (unsigned)W);
    const long long at = rstart[blockIdx.x], len = rlen[blockIdx.x];
    if (at < 0 || len < 0 || at > cap || len > cap - at) return;
    long long end = at + (len + kFxRun - 1) / kFxRun * kFxRun;
    end = end > cap ? cap : end;
    for (long long q = at + len + threadIdx.x; q < end; q += 256) { ent[q] = 0u; val[q] = 0.0f; }
    for (long long g = at / kFxRun + threadIdx.x; g < end / kFxRun; g += 256) tbase[g] = w << kFxWindowBits;
}

// largest m in [lo, hi] with ptr[m] <= e  (ptr[lo] <= e is given)
__device__ __forceinline__ long long fx_owner(const long long *__restrict__ ptr, long long lo, long long hi, long long e) {
    while (lo < hi) {
        const long long mid = lo + (hi - lo + 1) / 2;
        if (ptr[mid] <= e) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// The same, starting from a lower bound that is usually close: gallop upwards, then bisect.
__device__ __forceinline__ long long fx_owner_from(const long long *__restrict__ ptr, long long lo, long long M,
                                                   long long e) {
    long long step = 1, hi = lo;
    while (hi < M - 1) {
        const long long nxt = hi + step < M - 1 ? hi + step : M - 1;
        if (ptr[nxt] <= e) { lo = nxt; hi = nxt; step <<= 1; } else { hi = nxt - 1; break; }
    }
    return fx_owner(ptr, lo, hi < lo ? lo : hi, e);
}

// Stable split: entry e of the source layout goes to the next free place of its run.  One wave
// per tile (a tile lies in one window), 64 entries per step in source order; inside a step the
// lanes with the same panel are ranked by lane.
__global__ __launch_bounds__(256) void fx_scatter_kernel(const long long *__restrict__ ptr, long long M,
                                                         const int *__restrict__ idx, const float *__restrict__ val,
                                                         long long ntiles, int P, int W,
                                                         const long long *__restrict__ wsrc,
                                                         const long long *__restrict__ tfirst,
                                                         const long long *__restrict__ cnt,
                                                         const long long *__restrict__ shift, long long cap,
                                                         unsigned *__restrict__ ent, float *__restrict__ valo) {
    __shared__ long long cur[4][kFxMaxPanels];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long tile = blockIdx.x * 4LL + wave;
    long long e0 = 0, e1 = 0;
    int w = 0;
    if (tile < ntiles) {
        w = fx_tile_range(wsrc, tfirst, W, tile, &e0, &e1);
        for (int k = lane; k < P; k += 64) cur[wave][k] = cnt[(long long)k * ntiles + tile] + shift[k * W + w];
    }
    __syncthreads();
    if (tile >= ntiles || e0 >= e1) return;            // whole waves leave: no block-wide barrier below
    const unsigned long long lt = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    const long long wbase = (long long)w << kFxWindowBits;
    long long mprev = wbase < M - 1 ? wbase : M - 1;  // owners of this tile's entries start at the window's
    mprev = mprev < 0 ? 0 : mprev;
    for (long long eb = e0; eb < e1; eb += 64) {
        const long long e = eb + lane;
        const bool ok = e < e1;
        const long long elast = eb + 63 < e1 ? eb + 63 : e1 - 1;
        // owners (row of a CSR entry, column of a CSC entry): between those of the step's ends
        const long long m0 = fx_owner_from(ptr, mprev, M, eb);      // owners ascend with the entries
        const long long m1 = fx_owner_from(ptr, m0, M, elast);
        mprev = m1;
        const long long m = ok ? fx_owner(ptr, m0, m1, e) : m0;
        const int raw = ok ? idx[e] : 0;
        const unsigned key = min((unsigned)raw >> kFxPanelBits, (unsigned)(P - 1));
        long long pos = 0;
        unsigned long long todo = __ballot(ok);
        while (todo) {
            const int lead = __builtin_ctzll(todo);
            const unsigned kk = (unsigned)__builtin_amdgcn_readlane((int)key, lead);
            const unsigned long long same = __ballot(ok && key == kk);
            const long long base = cur[wave][kk];
            if (ok && key == kk) pos = base + __builtin_popcountll(same & lt);
            if (lane == lead) cur[wave][kk] = base + __builtin_popcountll(same);
            todo &= ~same;
        }
        if (ok && pos >= 0 && pos < cap) {
            const unsigned delta = (unsigned)(m - wbase) & ((1u << kFxWindowBits) - 1u);
            ent[pos] = ((unsigned)raw & (unsigned)(kFxPanel - 1)) | (delta << kFxPanelBits);
            valo[pos] = val[e];
        }
    }
}

// *slot = max(*slot, bits of max |x|); bits of non-negative floats order as unsigned integers
__global__ __launch_bounds__(256) void fx_absmax_kernel(const float *__restrict__ x, long long n,
                                                        unsigned *__restrict__ slot) {
    __shared__ unsigned red[256];
    unsigned m = 0;
    for (long long i = blockIdx.x * 256LL + threadIdx.x; i < n; i += (long long)gridDim.x * 256)
        m = max(m, __float_as_uint(x[i]) & 0x7FFFFFFFu);
    red[threadIdx.x] = m;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] = max(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    if (threadIdx.x == 0) atomicMax(slot, red[0]);
}

// *slot = max(*slot, longest run ptr[m + 1] - ptr[m]), capped at 2^31 - 1
__global__ __launch_bounds__(256) void fx_maxlen_kernel(const long long *__restrict__ ptr, long long M,
                                                        unsigned *__restrict__ slot) {
    __shared__ unsigned red[256];
    unsigned m = 0;
    for (long long i = blockIdx.x * 256LL + threadIdx.x; i < M; i += (long long)gridDim.x * 256) {
        const long long len = ptr[i + 1] - ptr[i];
        m = max(m, (unsigned)(len < 0 ? 0 : len > 0x7FFFFFFFLL ? 0x7FFFFFFFLL : len));
    }
    red[threadIdx.x] = m;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] = max(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    if (threadIdx.x == 0) atomicMax(slot, red[0]);
}

__global__ void fx_set_slots_kernel(unsigned *__restrict__ slots, int first, int count) {
    const int i = threadIdx.x;
    if (i < count) slots[first + i] = 0;
}

// ------------------------------------------------------------------ the pass

// Exponent e with |sum of maxlen products| * 2^e < 2^62, from the bit patterns of the largest
// |value| and the largest |element of the gathered vector|: |v| < 2^(ev + 1), |x| < 2^(ex + 1).
__device__ __forceinline__ int fx_exponent(unsigned maxval_bits, unsigned maxvec_bits, unsigned maxlen) {
    const int ev = (int)((maxval_bits >> 23) & 255u) - 127;
    const int ex = (int)((maxvec_bits >> 23) & 255u) - 127;
    const int cl = maxlen > 1 ? 32 - __clz((int)(maxlen - 1)) : 0;
    const int e = 60 - ev - ex - cl;
    return e < -126 ? -126 : e > 126 ? 126 : e;
}

// The layout is the library's own, but it lives in the caller's workspace: whatever that memory
// holds, panel starts are forced into [0, cap] and to multiples of four before they are used.
__device__ __forceinline__ long long fx_panel_start(const long long *__restrict__ pstart, int p, long long cap) {
    const long long s = pstart[p] & ~3LL;
    return s < 0 ? 0 : s > cap ? cap : s;
}

__global__ __launch_bounds__(kFxThreads) void fx_pass_kernel(
    const unsigned *__restrict__ ent, const float *__restrict__ val, const int *__restrict__ tbase,
    const float *__restrict__ vec, long long vec_len, long long cap, const long long *__restrict__ pstart,
    int P, long long span, unsigned *slots, int vec_slot, int len_slot, int e_slot, long long *__restrict__ part) {
    extern __shared__ unsigned long long fx_sums[];    // [kFxPanel]
    const int tid = threadIdx.x;
    const int e2 = fx_exponent(slots[kFxSlotMaxVal], slots[vec_slot], slots[len_slot]);
    if (blockIdx.x == 0 && tid == 0) slots[e_slot] = (unsigned)e2;          // for the kernel that converts back
    const float scale = __builtin_ldexpf(1.0f, e2);
    const unsigned vmax = (unsigned)(vec_len - 1);
    const long long total = fx_panel_start(pstart, P, cap);
    const long long r0 = (long long)blockIdx.x * span;
    const long long r1 = r0 + span < total ? r0 + span : total;
    if (r0 >= total) return;                           // uniform over the block
    // first panel of the span: the last p with pstart[p] <= r0 (the same for every thread)
    int p = 0;
    {
        int lo = 0, hi = P - 1;
        while (lo < hi) {
            const int mid = lo + (hi - lo + 1) / 2;
            if (fx_panel_start(pstart, mid, cap) <= r0) lo = mid; else hi = mid - 1;
        }
        p = lo;
    }
    typedef float f4 __attribute__((ext_vector_type(4)));
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    const u4 *__restrict__ e4p = reinterpret_cast<const u4 *>(ent);
    const f4 *__restrict__ v4p = reinterpret_cast<const f4 *>(val);
    const long long stride = (long long)kFxThreads * kFxUnroll;
    for (; p < P; ++p) {
        const long long s0 = fx_panel_start(pstart, p, cap), s1 = fx_panel_start(pstart, p + 1, cap);
        if (s0 >= r1) break;
        const long long b0 = s0 > r0 ? s0 : r0, b1 = s1 < r1 ? s1 : r1;
        if (b1 <= b0) continue;                        // an empty panel (or a start out of order)
        for (int i = tid; i < kFxPanel; i += kFxThreads) fx_sums[i] = 0ull;
        __syncthreads();
        // Two loads stand between an entry and its sum: the entry itself, then the element of the
        // other vector it points at.  The entries of the next round are requested before the current
        // round's elements are waited for, so that one latency is paid per round, not two.  A lane
        // takes four consecutive entries with one 16-byte load per array; the 4096 entries the block
        // takes in one step are one group of the layout (b0 is a multiple of 4096: runs are padded,
        // spans are multiples of 4096) and share the start of their window.
        u4 g[kFxUnroll]; f4 v[kFxUnroll]; unsigned wb[kFxUnroll];
#define SLAQ_FX_LOAD(Q)                                                                      \
    _Pragma("unroll") for (int u = 0; u < kFxUnroll; ++u) {                                  \
        const long long q_ = (Q) + (long long)u * kFxThreads;                                \
        const bool ok_ = q_ < q1;                                                            \
        g[u] = ok_ ? __builtin_nontemporal_load(e4p + q_) : u4{0u, 0u, 0u, 0u};              \
        v[u] = ok_ ? __builtin_nontemporal_load(v4p + q_) : f4{0.0f, 0.0f, 0.0f, 0.0f};      \
        wb[u] = ok_ ? (unsigned)tbase[q_ >> 10] : 0u;                                        \
    }
        const long long q1 = b1 >> 2;
        long long q = (b0 >> 2) + tid;
        if (q < q1) SLAQ_FX_LOAD(q)
        for (; q < q1; q += stride) {
            f4 x[kFxUnroll], vv[kFxUnroll]; u4 ll[kFxUnroll];
#pragma unroll
            for (int u = 0; u < kFxUnroll; ++u) {
                // keep every index inside its array whatever the memory holds
#pragma unroll
                for (int c = 0; c < 4; ++c) x[u][c] = vec[min(wb[u] + (g[u][c] >> kFxPanelBits), vmax)];
                vv[u] = v[u]; ll[u] = g[u];
            }
            if (q + stride < q1) SLAQ_FX_LOAD(q + stride)
#pragma unroll
            for (int u = 0; u < kFxUnroll; ++u) {
                if (q + (long long)u * kFxThreads < q1) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const long long t = __float2ll_rn((vv[u][c] * x[u][c]) * scale);
                        atomicAdd(&fx_sums[ll[u][c] & (unsigned)(kFxPanel - 1)], (unsigned long long)t);
                    }
                }
            }
        }
#undef SLAQ_FX_LOAD
        __syncthreads();
        // slice blockIdx + p: both count upwards along the stream, so the slices of a panel are
        // neighbours and no two (block, panel) pairs share one
        long long *__restrict__ dst = part + ((long long)blockIdx.x + p) * kFxPanel;
        for (int i = tid; i < kFxPanel; i += kFxThreads) dst[i] = (long long)fx_sums[i];
        __syncthreads();
    }
}

// out[i] = (sum over the slices of i's panel) * 2^-e.  A block takes 256 outputs, 32 at a time;
// its eight groups of 32 lanes share the slices (a popular panel has hundreds), integer sums in
// any order.
__global__ __launch_bounds__(256) void fx_finish_kernel(const long long *__restrict__ part,
                                                        const long long *__restrict__ pstart, int P, long long span,
                                                        long long cap, long long out_len,
                                                        const unsigned *__restrict__ slots, int e_slot,
                                                        float *__restrict__ out) {
    __shared__ long long red[8][8][32];
    const int o32 = threadIdx.x & 31, sl = threadIdx.x >> 5;
    const long long base = blockIdx.x * 256LL;                 // 256 divides the panel: a block is in one panel
    if (base >= out_len) return;
    const int p = (int)(base / kFxPanel);
    // the blocks whose spans meet the panel's entries [s0, s1): floor(s0 / span) .. floor((s1 - 1) / span)
    const long long s0 = fx_panel_start(pstart, p, cap), s1 = fx_panel_start(pstart, p + 1, cap);
    const long long c0 = s0 / span + p, c1 = s1 > s0 ? (s1 - 1) / span + p + 1 : c0;
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        const long long i = base + g * 32 + o32;
        const int o = (int)(i - (long long)p * kFxPanel);
        long long s = 0;
        if (i < out_len) {
            // four independent loads in flight per lane
            long long s1 = 0, s2 = 0, s3 = 0, c = c0 + sl;
            for (; c + 24 < c1; c += 32) {
                s += part[c * kFxPanel + o];
                s1 += part[(c + 8) * kFxPanel + o];
                s2 += part[(c + 16) * kFxPanel + o];
                s3 += part[(c + 24) * kFxPanel + o];
            }
            for (; c < c1; c += 8) s += part[c * kFxPanel + o];
            s += (s1 + s2) + s3;
        }
        red[g][sl][o32] = s;
    }
    __syncthreads();
    // thread t finishes output base + t
    const long long i = base + threadIdx.x;
    if (i < out_len) {
        const int g = threadIdx.x >> 5;
        long long s = 0;
        for (int q = 0; q < 8; ++q) s += red[g][q][o32];
        out[i] = (float)ldexp((double)s, -(int)slots[e_slot]);
    }
}

hipError_t fx_build_pass(const FxPass &ps, const long long *ptr, long long M, const int *idx, const float *val,
                         long long nnz, long long *cnt, long long *bsum, hipStream_t st) {
    hipError_t e;
    const long long ntiles = ps.ntiles;
    const unsigned tb = (unsigned)((ntiles + 3) / 4);
    hipLaunchKernelGGL(fx_tiles_kernel, dim3(1), dim3(64), 0, st, ptr, M, nnz, ps.W, ps.wsrc, ps.tfirst);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fx_hist_kernel, dim3(tb), dim3(256), 0, st, idx, ntiles, ps.P, ps.W, ps.wsrc, ps.tfirst, cnt);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const long long n = (long long)ps.P * ntiles;
    const long long nb = (n + kScanBlock - 1) / kScanBlock;
    hipLaunchKernelGGL(fx_scan_block_kernel, dim3((unsigned)nb), dim3(256), 0, st, cnt, n, bsum);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fx_scan_tops_kernel, dim3(1), dim3(64), 0, st, nb, bsum);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fx_scan_add_kernel, dim3((unsigned)((n + 1 + 255) / 256)), dim3(256), 0, st, n, bsum, nb, cnt);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fx_pstart_kernel, dim3(1), dim3(64), 0, st, cnt, ntiles, ps.P, ps.W, ps.tfirst, ps.pstart, ps.shift,
                       ps.rstart, ps.rlen);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fx_pad_kernel, dim3((unsigned)(ps.P * ps.W)), dim3(256), 0, st, ps.W, ps.cap, ps.rstart, ps.rlen,
                       ps.ent, ps.val, ps.tbase);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fx_scatter_kernel, dim3(tb), dim3(256), 0, st, ptr, M, idx, val, ntiles, ps.P, ps.W, ps.wsrc,
                       ps.tfirst, cnt, ps.shift, ps.cap, ps.ent, ps.val);
    return hipGetLastError();
}

}  // namespace

// Which passes take this path, with how many panels and blocks.  A function of the shape alone.
void sparse_fx_plan(long long N, long long D, long long nnz, FxPass *row, FxPass *col) {
    FxPass *ps[2] = {row, col};
    const long long out_len[2] = {N, D}, gather_len[2] = {D, N};
    for (int i = 0; i < 2; ++i) {
        FxPass &f = *ps[i];
        f = FxPass{};
        f.out_len = out_len[i];
        f.gather_len = gather_len[i];
        const long long P = (out_len[i] + kFxPanel - 1) / kFxPanel;
        const long long W = (gather_len[i] + (1LL << kFxWindowBits) - 1) >> kFxWindowBits;
        // enough entries that the padding of the P W runs (less than 4096 each) stays under a quarter
        f.on = nnz >= kFxMinEntries && P <= kFxMaxPanels && W <= kFxMaxWindows && nnz >= 4 * kFxRun * P * W;
        if (!f.on) continue;
        f.P = (int)P;
        f.W = (int)W;
        f.cap = ((nnz + kFxRun - 1) / kFxRun + P * W) * kFxRun;
        // one block per compute unit at most, each with an equal share of the padded stream,
        // whatever the sizes of the panels
        const long long span = ((f.cap + kFxBlocks - 1) / kFxBlocks + kFxRun - 1) / kFxRun * kFxRun;
        f.span = span < 32768 ? 32768 : span;
        f.blocks = (int)((f.cap + f.span - 1) / f.span);
        f.slices = f.blocks + P;
        f.ntiles = (nnz + kFxTile - 1) / kFxTile + W;       // no tile crosses the start of a window
    }
}

// Once per matrix: both layouts, the largest |value| and the longest row and column.
hipError_t launch_sparse_fx_build(const SparseArgs &a, const SparseFx &fx, hipStream_t st) {
    hipError_t e;
    hipLaunchKernelGGL(fx_set_slots_kernel, dim3(1), dim3(64), 0, st, fx.slots, 0, kFxSlots);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fx_absmax_kernel, dim3(1024), dim3(256), 0, st, a.row_val, a.nnz, fx.slots + kFxSlotMaxVal);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fx_maxlen_kernel, dim3(1024), dim3(256), 0, st, a.row_ptr, a.N, fx.slots + kFxSlotLenRow);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fx_maxlen_kernel, dim3(1024), dim3(256), 0, st, a.col_ptr, a.D, fx.slots + kFxSlotLenCol);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // row pass: outputs are rows, source is the column layout (columns ascend inside a panel)
    if (fx.row.on &&
        (e = fx_build_pass(fx.row, a.col_ptr, a.D, a.row_idx, a.col_val, a.nnz, fx.cnt, fx.bsum, st)) != hipSuccess)
        return e;
    // column pass: outputs are columns, source is the row layout
    if (fx.col.on &&
        (e = fx_build_pass(fx.col, a.row_ptr, a.N, a.col_idx, a.row_val, a.nnz, fx.cnt, fx.bsum, st)) != hipSuccess)
        return e;
    return hipSuccess;
}

// At the start of every call: the largest |w| of the entering iterate, no residuals yet.
hipError_t launch_sparse_fx_begin(const SparseArgs &a, const SparseFx &fx, hipStream_t st) {
    hipError_t e;
    hipLaunchKernelGGL(fx_set_slots_kernel, dim3(1), dim3(64), 0, st, fx.slots, kFxSlotMaxW, 2);   // max|w|, max|r|
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fx_absmax_kernel, dim3(256), dim3(256), 0, st, a.w, a.D, fx.slots + kFxSlotMaxW);
    return hipGetLastError();
}

// z = X w (row = true, into out [N]) or s = X^T r (row = false, into out [D])
hipError_t launch_sparse_fx_pass(const SparseFx &fx, bool row, const float *vec, long long vec_len, long long nnz,
                                 float *out, hipStream_t st) {
    const FxPass &ps = row ? fx.row : fx.col;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fx_pass_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kFxPanel * 8);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fx_pass_kernel, dim3((unsigned)ps.blocks), dim3(kFxThreads), kFxPanel * 8, st, ps.ent, ps.val,
                       ps.tbase, vec, vec_len, ps.cap, ps.pstart, ps.P, ps.span, fx.slots,
                       row ? kFxSlotMaxW : kFxSlotMaxR, row ? kFxSlotLenRow : kFxSlotLenCol,
                       row ? kFxSlotERow : kFxSlotECol, ps.part);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(fx_finish_kernel, dim3((unsigned)((ps.out_len + 255) / 256)), dim3(256), 0, st, ps.part, ps.pstart,
                       ps.P, ps.span, ps.cap, ps.out_len, fx.slots, row ? kFxSlotERow : kFxSlotECol, out);
    return hipGetLastError();
}

}  // namespace slaqglm
