// K-Means (Lloyd) iteration for gfx950.
//
//   shift      : once per call, the column means of a sample of the rows; the assignment works
//                on points and centroids minus this shift (distances are unchanged, the fp32
//                rounding of the expanded form is not: it scales with |x|^2 + |c|^2).
//   center     : Cc = C - shift, cn[k] = |Cc_k|^2 (fp32), +inf for the padding slots past K.
//   assign     : the nearest centroid minimises cn[k] - 2 x_i . c_k (the |x_i|^2 term is common to
//                all k), lowest index on equal values.  Three kernels, by shape: few centroids
//                (K <= 32, or K <= 64 and K D <= 4096) on the vector units, a row per lane;
//                otherwise D <= 128 with operands
//                split into bfloat16 parts on the matrix cores, centroids stationary in
//                registers; otherwise per tile of TR points held in LDS, 64 centroids at a time
//                (v_mfma_f32_32x32x2_f32, fp32 in, fp32 accumulate).  The squared distance that
//                enters the loss is recomputed for the chosen centroid as sum_j (x_ij - c_kj)^2,
//                which has no cancellation: by the two matrix-core kernels themselves (the tile
//                is still in LDS), by the accumulation pass for the first (whose rows are gone).
//   accumulate : second pass over X.  A wave owns a slab of 64 columns, a contiguous range of
//                rows and up to 32 clusters, keeps their sums in registers and adds the rows
//                assigned to them in row order.  Partials go to part[split].
//   finalize   : per centroid and 16 columns, adds the partials in a fixed order (fp64: sixteen
//                interleaved runs over the splits, then the runs), divides by the cluster size
//                (an empty cluster keeps its centroid), and sums the loss partials.
//
// Lane layout of the 32x32x2 instruction (lane l of 64): A[i][k] from lane i + 32 k,
// B[k][j] from lane j + 32 k, D[i][j] in lane j + 32 ((i / 4) % 2), register (i % 4) + 4 (i / 8).
#include "kmeans_internal.h"

#include <limits>

namespace slaqglm {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kWLd4 = 9;                   // LDS row stride of the centroid piece in float4 (32 + 4 floats)
constexpr size_t kLdsBudget = 150 * 1024;  // of the 160 KB of a compute unit

static size_t assign_lds_bytes(int TR, int Dp) {
    return sizeof(f4) * ((size_t)TR * (Dp / 4 + 1) + kKmChunk * kWLd4) + sizeof(int) * TR + sizeof(float) * 8;
}

KmShape km_shape(long long N, int D, int K) {
    KmShape s;
    s.small = K <= 32 || (K <= kKmSmallK && (long long)K * D <= kKmSmallWork);
    s.split = !s.small && D <= kKmSplitMaxD;
    s.Dp = s.split ? (D + 63) / 64 * 64 : (D + 31) / 32 * 32;
    s.Kp = s.split ? (K + 255) / 256 * 256 : (K + kKmChunk - 1) / kKmChunk * kKmChunk;
    s.TR = s.small ? kKmSmallRows : s.split ? 32 : 128;
    while (!s.small && !s.split && s.TR > 32 && assign_lds_bytes(s.TR, s.Dp) > kLdsBudget) s.TR /= 2;
    s.T = (N + s.TR - 1) / s.TR;
    s.lds_assign = (s.small || s.split) ? 0 : assign_lds_bytes(s.TR, s.Dp);
    // split path: a fixed grid of persistent blocks (one per compute unit), contiguous tile ranges
    s.tiles_per_block = (s.T + 255) / 256;
    s.stream_blocks = (int)((s.T + s.tiles_per_block - 1) / s.tiles_per_block);     // no block without tiles
    s.nslab = (D + 63) / 64;
    s.G = (K + 31) / 32;
    // row splits: at most 1024, at least 1024 rows each, and at most 1 GiB of partial sums
    long long pmax = 1024;
    const long long owners = (long long)s.G * s.nslab;                // waves per row split
    if (owners * pmax < 8192) pmax = (8192 + owners - 1) / owners;    // few owners: more splits keep enough rows in flight
    const long long cap = (1LL << 28) / ((long long)K * D);
    if (pmax > cap) pmax = cap < 1 ? 1 : cap;
    long long rps = (N + pmax - 1) / pmax;
    if (rps < 1024) rps = 1024;
    rps = (rps + 63) / 64 * 64;
    s.rows_per_split = rps;
    s.P = (int)((N + rps - 1) / rps);
    // loss partials: one per wave of the accumulation pass (few centroids), else per wave of the
    // streaming assignment or per tile
    s.lossN = s.small ? owners * s.P : s.split ? (long long)s.stream_blocks * 8 : s.T;
    return s;
}

__device__ __forceinline__ floatx16 km_mfma(float a, float b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// The common shift: column means over at most 1024 evenly spaced rows.  Distances do not change
// when the points and the centroids are shifted together, but the fp32 rounding of the expanded
// form |c|^2 - 2 x . c scales with |x|^2 + |c|^2, so data far from the origin would lose the
// near ties; after the shift both are of the size of the data's spread.  One slice of the
// sample per wave, the sixteen waves added in order.  Values that are not finite are left out, so
// that one bad row cannot spoil the shift of all the others.
constexpr int kKmMeanSample = 1024;
constexpr int kKmMeanWaves = 16;

__global__ __launch_bounds__(64 * kKmMeanWaves) void kmeans_mean_kernel(const float *__restrict__ X, long long N, int D,
                                                                        float *__restrict__ mean) {
    __shared__ float red[kKmMeanWaves][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + lane;
    const long long S = N < kKmMeanSample ? N : kKmMeanSample;
    const long long stride = N / S;
    float s = 0.0f;
    if (col < D) {
        // sample rows wave, wave + 16, ...: eight loads in flight, added in order
        long long i = wave;
        for (; i + 7 * kKmMeanWaves < S; i += 8 * kKmMeanWaves) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = X[(size_t)((i + u * kKmMeanWaves) * stride) * D + col];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += __builtin_isfinite(v[u]) ? v[u] : 0.0f;
        }
        for (; i < S; i += kKmMeanWaves) {
            const float v = X[(size_t)(i * stride) * D + col];
            s += __builtin_isfinite(v) ? v : 0.0f;
        }
    }
    red[wave][lane] = s;
    __syncthreads();
    if (wave == 0 && col < D) {
        float t = red[0][lane];
        for (int w = 1; w < kKmMeanWaves; ++w) t += red[w][lane];
        t /= (float)S;
        mean[col] = __builtin_isfinite(t) ? t : 0.0f;      // any finite shift is valid; NaN or inf is not
    }
}

// Cc = C - mean, cn[k] = |Cc_k|^2 (+inf for the padding slots past K): one wave per centroid.
__global__ __launch_bounds__(256) void kmeans_center_kernel(const float *__restrict__ C, const float *__restrict__ mean,
                                                            int D, int K, int Kp, float *__restrict__ Cc,
                                                            float *__restrict__ cn) {
    const int lane = threadIdx.x & 63;
    const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (k >= Kp) return;
    float s = 0.0f;
    if (k < K)
        for (int j = lane; j < D; j += 64) {
            const float c = C[(size_t)k * D + j] - mean[j];
            Cc[(size_t)k * D + j] = c;
            s = __builtin_fmaf(c, c, s);
        }
    for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) cn[k] = k < K ? s : std::numeric_limits<float>::infinity();
}

template <int TR>
__global__ __launch_bounds__(TR * 2) void kmeans_assign_kernel(
    const float *__restrict__ X, const float *__restrict__ C, const float *__restrict__ mean,
    const float *__restrict__ cn, long long N, int D, int K, int Dp, int Kp, int *__restrict__ assign,
    float *__restrict__ lossP) {
    constexpr int NT = TR * 2;             // threads: one wave per 32 rows
    constexpr int NW = TR / 32;
    constexpr int Q = kKmChunk * 8 / NT;   // float4 of a 64 x 32 centroid piece staged per thread
    extern __shared__ f4 km_smem[];
    const int ldx4 = Dp / 4 + 1;           // odd stride in float4: rows fall in different banks
    f4 *Xs4 = km_smem;                     // [TR][ldx4]
    f4 *Ws4 = Xs4 + (size_t)TR * ldx4;     // [64][9]
    int *rowk = reinterpret_cast<int *>(Ws4 + kKmChunk * kWLd4);   // [TR]
    float *wsum = reinterpret_cast<float *>(rowk + TR);            // [NW]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;
    const long long r0 = (long long)blockIdx.x * TR;
    const int D4 = D >> 2, Dp4 = Dp >> 2;
    const f4 *__restrict__ X4 = reinterpret_cast<const f4 *>(X);
    const f4 *__restrict__ C4 = reinterpret_cast<const f4 *>(C);
    const f4 *__restrict__ M4 = reinterpret_cast<const f4 *>(mean);

    // the tile of points minus the common shift, zero beyond D and beyond N
    for (int idx = tid; idx < TR * Dp4; idx += NT) {
        const int row = idx / Dp4, c4 = idx - row * Dp4;
        const long long r = r0 + row;
        f4 v = {0.0f, 0.0f, 0.0f, 0.0f};
        if (r < N && c4 < D4) v = __builtin_nontemporal_load(X4 + r * D4 + c4) - M4[c4];
        Xs4[row * ldx4 + c4] = v;
    }

    const int nK = Dp / 32, nC = Kp / kKmChunk;
    const int steps = nC * nK;
    floatx16 acc0 = {0}, acc1 = {0};
    float bv[16]; int bk[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) { bv[r] = std::numeric_limits<float>::infinity(); bk[r] = 0; }

    // piece (c, kc) = centroids 64 c .. 64 c + 63, columns 32 kc .. 32 kc + 31; slots outside
    // [K, D] read a valid address and are multiplied by zero
#define SLAQ_KM_FETCH(CC, KC)                                                                \
    {                                                                                        \
        _Pragma("unroll") for (int q = 0; q < Q; ++q) {                                      \
            const int idx = tid + NT * q;                                                    \
            const int cent = (CC) * kKmChunk + (idx >> 3);                                   \
            const int col4 = (KC) * 8 + (idx & 7);                                           \
            const bool ok = cent < K && col4 < D4;                                           \
            wm[q] = ok ? 1.0f : 0.0f;                                                        \
            wr[q] = C4[(size_t)(cent < K ? cent : 0) * D4 + (col4 < D4 ? col4 : 0)];         \
        }                                                                                    \
    }
#define SLAQ_KM_STASH()                                                                      \
    {                                                                                        \
        _Pragma("unroll") for (int q = 0; q < Q; ++q) {                                      \
            const int idx = tid + NT * q;                                                    \
            Ws4[(idx >> 3) * kWLd4 + (idx & 7)] = wr[q] * wm[q];                             \
        }                                                                                    \
    }
    {
        f4 wr[Q]; float wm[Q];
        SLAQ_KM_FETCH(0, 0)
        SLAQ_KM_STASH()
    }
    __syncthreads();

    int c = 0, kc = 0;
    for (int step = 0; step < steps; ++step) {
        int c2 = c, kc2 = kc + 1;
        if (kc2 == nK) { kc2 = 0; c2 = c + 1; }
        if (step + 1 >= steps) { c2 = c; kc2 = kc; }    // last trip re-reads its own piece (cache hit)
        f4 wr[Q]; float wm[Q];
        SLAQ_KM_FETCH(c2, kc2)
        __builtin_amdgcn_sched_barrier(0);              // keep the prefetch ahead of the matrix ops
        const f4 *arow = Xs4 + (wave * 32 + li) * ldx4 + kc * 8 + lh;
        const f4 *b0row = Ws4 + li * kWLd4 + lh;
        const f4 *b1row = Ws4 + (32 + li) * kWLd4 + lh;
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {                // 8 columns: lanes lh = 0 take 0..3, lh = 1 take 4..7
            const f4 a = arow[2 * kb];
            const f4 b0 = b0row[2 * kb];
            const f4 b1 = b1row[2 * kb];
            acc0 = km_mfma(a.x, b0.x, acc0); acc1 = km_mfma(a.x, b1.x, acc1);
            acc0 = km_mfma(a.y, b0.y, acc0); acc1 = km_mfma(a.y, b1.y, acc1);
            acc0 = km_mfma(a.z, b0.z, acc0); acc1 = km_mfma(a.z, b1.z, acc1);
            acc0 = km_mfma(a.w, b0.w, acc0); acc1 = km_mfma(a.w, b1.w, acc1);
        }
        if (kc == nK - 1) {
            // chunk c is complete: this lane holds centroids 64 c + li (acc0) and 64 c + 32 + li
            // (acc1) for 16 of the wave's rows; chunks arrive in increasing index order and the
            // comparisons are strict, so equal values keep the lower index
            const int k0 = c * kKmChunk + li, k1 = k0 + 32;
            const float cn0 = cn[k0], cn1 = cn[k1];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float v0 = __builtin_fmaf(-2.0f, acc0[r], cn0);
                const float v1 = __builtin_fmaf(-2.0f, acc1[r], cn1);
                if (v0 < bv[r]) { bv[r] = v0; bk[r] = k0; }
                if (v1 < bv[r]) { bv[r] = v1; bk[r] = k1; }
                acc0[r] = 0.0f; acc1[r] = 0.0f;
            }
        }
        __syncthreads();
        SLAQ_KM_STASH()
        __syncthreads();
        c = c2; kc = kc2;
    }
#undef SLAQ_KM_FETCH
#undef SLAQ_KM_STASH

    // nearest centroid of each row: minimum over the 32 lanes that share lh, lower index on ties
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        float v = bv[r]; int k = bk[r];
#pragma unroll
        for (int o = 1; o <= 16; o <<= 1) {
            const float ov = __shfl_xor(v, o, 64);
            const int ok = __shfl_xor(k, o, 64);
            if (ov < v || (ov == v && ok < k)) { v = ov; k = ok; }
        }
        if (li == 0) rowk[wave * 32 + 8 * (r >> 2) + 4 * lh + (r & 3)] = k;
    }
    __syncthreads();

    // squared distance to the chosen centroid, straight from the definition; two threads per row
    const int row = tid >> 1, half = tid & 1;
    const int a = rowk[row];
    float d = 0.0f;
    for (int j4 = half * (Dp4 / 2); j4 < (half + 1) * (Dp4 / 2); ++j4) {
        const f4 x = Xs4[row * ldx4 + j4];
        f4 cc = {0.0f, 0.0f, 0.0f, 0.0f};
        if (j4 < D4) cc = C4[(size_t)a * D4 + j4];
        const f4 t = x - cc;
        d = __builtin_fmaf(t.x, t.x, d); d = __builtin_fmaf(t.y, t.y, d);
        d = __builtin_fmaf(t.z, t.z, d); d = __builtin_fmaf(t.w, t.w, d);
    }
    d = d + __shfl_xor(d, 1, 64);
    const bool valid = r0 + row < N;
    if (half == 0 && valid) assign[r0 + row] = a;
    float v = (half == 0 && valid) ? d : 0.0f;
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    if (lane == 0) wsum[wave] = v;
    __syncthreads();
    if (tid == 0) {
        float s = wsum[0];
        for (int w = 1; w < NW; ++w) s += wsum[w];
        lossP[blockIdx.x] = s;
    }
}

// ---- Assignment for few centroids (K <= 32, or K <= 64 with K D <= 4096) --------------------
//
// With so few centroids a matrix tile would be mostly padding, and the products are cheap
// enough for the vector units: a lane owns a row and keeps x_i . c_k for every k in registers.
// The centroid values are the same for all lanes, so they arrive through the scalar data path
// (read-only) and cost no vector register or LDS traffic.  The rows reach their lanes through
// LDS: 32 columns of 256 rows at a time, loaded so that eight lanes read one row's 128 bytes,
// stored with an odd row stride.
constexpr int kSmCols = 32;
constexpr int kSmLd = kSmCols + 1;

template <int KG>                         // groups of eight centroids: K <= 8 KG
__global__ __launch_bounds__(kKmSmallRows) void kmeans_assign_small_kernel(
    const float *__restrict__ X, const float *__restrict__ C, const float *__restrict__ mean,
    const float *__restrict__ cn, long long N, int D, int K, int *__restrict__ assign) {
    __shared__ float xs[kKmSmallRows * kSmLd];
    const int tid = threadIdx.x;
    const long long r0 = (long long)blockIdx.x * kKmSmallRows;
    const int rows = (int)((N - r0) < kKmSmallRows ? (N - r0) : kKmSmallRows);
    const int D4 = D >> 2;
    const f4 *__restrict__ X4 = reinterpret_cast<const f4 *>(X) + r0 * D4;
    const f4 *__restrict__ C4 = reinterpret_cast<const f4 *>(C);
    const f4 *__restrict__ M4 = reinterpret_cast<const f4 *>(mean);
    const int nch = (D + kSmCols - 1) / kSmCols;

    float acc[8 * KG];
#pragma unroll
    for (int k = 0; k < 8 * KG; ++k) acc[k] = 0.0f;

    // piece ch of the tile: thread t brings float4 number (t & 7) of rows (t >> 3) + 32 q
    f4 pre[8], mpre;                      // mpre: the common shift of this thread's four columns
#define SLAQ_SM_FETCH(CH)                                                                    \
    {                                                                                        \
        const int c4_ = (CH) * (kSmCols / 4) + (tid & 7);                                    \
        mpre = f4{0.0f, 0.0f, 0.0f, 0.0f};                                                   \
        if (c4_ < D4) mpre = M4[c4_];                                                        \
        _Pragma("unroll") for (int q = 0; q < 8; ++q) {                                      \
            const int row_ = (tid >> 3) + 32 * q;                                            \
            f4 v_ = {0.0f, 0.0f, 0.0f, 0.0f};                                                \
            if (row_ < rows && c4_ < D4) v_ = X4[(size_t)row_ * D4 + c4_];                   \
            pre[q] = v_;                                                                     \
        }                                                                                    \
    }
    SLAQ_SM_FETCH(0);
    for (int ch = 0; ch < nch; ++ch) {
        if (ch) __syncthreads();                       // the previous piece has been read
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float *dst = xs + ((tid >> 3) + 32 * q) * kSmLd + 4 * (tid & 7);
            // the shift comes off here, where the prefetched values are first needed (columns past
            // D hold zero in both; rows past N are never written out)
            const f4 v = pre[q] - mpre;
            dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3];
        }
        __syncthreads();
        if (ch + 1 < nch) SLAQ_SM_FETCH(ch + 1);
        float x[kSmCols];
#pragma unroll
        for (int j = 0; j < kSmCols; ++j) x[j] = xs[tid * kSmLd + j];
        // Straight-line body: the scalar loads of a group of eight centroids go out together and
        // the next group's can be issued under this group's arithmetic.  Columns past D hold
        // x = 0 and re-read the last column; slots past K re-read the last centroid (never
        // chosen: the argmin below stops at K).
#pragma unroll
        for (int jg = 0; jg < kSmCols / 4; ++jg) {
            const int col4 = ch * (kSmCols / 4) + jg < D4 ? ch * (kSmCols / 4) + jg : D4 - 1;
#pragma unroll
            for (int g = 0; g < KG; ++g) {
                f4 c[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) c[u] = C4[(size_t)(8 * g + u < K ? 8 * g + u : K - 1) * D4 + col4];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    float a = acc[8 * g + u];
                    a = __builtin_fmaf(x[4 * jg], c[u][0], a);
                    a = __builtin_fmaf(x[4 * jg + 1], c[u][1], a);
                    a = __builtin_fmaf(x[4 * jg + 2], c[u][2], a);
                    a = __builtin_fmaf(x[4 * jg + 3], c[u][3], a);
                    acc[8 * g + u] = a;
                }
            }
        }
    }
#undef SLAQ_SM_FETCH
    float bv = std::numeric_limits<float>::infinity();
    int bk = 0;
#pragma unroll
    for (int k = 0; k < 8 * KG; ++k) {
        if (k < K) {
            const float v = __builtin_fmaf(-2.0f, acc[k], cn[k]);
            if (v < bv) { bv = v; bk = k; }
        }
    }
    if (tid < rows) assign[r0 + tid] = bk;
}

// ---- Assignment with split operands (D <= 128) ---------------------------------------------
//
// An fp32 value is the exact sum of three bfloat16 values (8 + 8 + 8 significant bits, same
// exponent range), x = xh + xm + xl.  The product x . c is then the sum of nine bfloat16 products,
// of which the six largest (xh ch, xm ch, xh cm, xl ch, xm cm, xh cl) carry everything down to
// 2^-24 relative: the same accuracy class as an fp32 dot product.  Each of them is exact in fp32
// and accumulates in fp32 on the matrix cores with v_mfma_f32_32x32x16_bf16, whose rate is 16
// times that of the fp32 instruction, so the six cost 3/8 of one fp32 product.
// Lane layout of the instruction (checked on the device): A[i][8 g .. 8 g + 7] in lane i + 32 g,
// B[8 g .. 8 g + 7][j] in lane j + 32 g, D as for the other 32x32 variants.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u4 __attribute__((ext_vector_type(4)));

constexpr int kSpK = 64;                   // the split path pads D to a multiple of this

// bfloat16 bit patterns (in the high halves) of the three parts of x
__device__ __forceinline__ void split3(float x, unsigned &h, unsigned &m, unsigned &l) {
    h = __float_as_uint(x) & 0xFFFF0000u;
    const float r = x - __uint_as_float(h);            // exact
    m = __float_as_uint(r) & 0xFFFF0000u;
    const float r2 = r - __uint_as_float(m);           // exact, at most 8 significant bits
    l = __float_as_uint(r2) & 0xFFFF0000u;
}

// Cs[part][k][j] (bfloat16 bits), part = 0, 1, 2; zero for k >= K or j >= D
__global__ __launch_bounds__(256) void kmeans_split_kernel(const float *__restrict__ C, int D, int K, int Kp, int Dp,
                                                           unsigned short *__restrict__ Cs) {
    const long long idx = blockIdx.x * 256LL + threadIdx.x;
    if (idx >= (long long)Kp * Dp) return;
    const int k = (int)(idx / Dp), j = (int)(idx - (long long)k * Dp);
    const float c = (k < K && j < D) ? C[(size_t)k * D + j] : 0.0f;
    unsigned h, m, l;
    split3(c, h, m, l);
    const size_t plane = (size_t)Kp * Dp;
    Cs[idx] = (unsigned short)(h >> 16);
    Cs[plane + idx] = (unsigned short)(m >> 16);
    Cs[2 * plane + idx] = (unsigned short)(l >> 16);
}

__device__ __forceinline__ floatx16 km_mfma_bf16(u4 a, u4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// The centroids stay put and the points stream: a block of 8 waves holds one group of 256
// centroids (32 per wave, as split A operands in registers, for the whole kernel) and walks over
// its share of the points in tiles of 32 rows.  The 512 threads load the next tile, split it and
// store the three parts in LDS as B operands; every wave multiplies its 32 centroids with the 32
// rows; the nearest centroid of a row is the minimum over a lane's 16 registers, its partner lane
// and the 8 waves (through LDS).  One barrier per tile: the tile after the next is in flight
// from HBM, the next tile is being written to LDS, and the distance of the previous tile's rows to
// their chosen centroids (rebuilt exactly from the parts still in LDS) is computed while the
// matrix cores work on the current one.  With more than 256 centroids the kernel runs once per
// group and carries the best value and index of every row in global memory.
// NKP = Dp / 64.
constexpr int kStWaves = 8;
constexpr int kStRows = 32;
constexpr int kStGroup = 32 * kStWaves;    // centroids per launch

template <int NKP>
__global__ __launch_bounds__(512) void kmeans_assign_stream_kernel(
    const float *__restrict__ X, const float *__restrict__ C, const float *__restrict__ mean,
    const unsigned short *__restrict__ Cs, const float *__restrict__ cn, long long N, int D, int Kp, int gbase,
    int first, int last,
    long long tiles, long long tiles_per_block, int *__restrict__ assign, float *__restrict__ bestv,
    float *__restrict__ lossW) {
    constexpr int Dp = kSpK * NKP;
    constexpr int NS = 4 * NKP;            // 16-column steps
    constexpr int RowB = 2 * Dp + 16;      // bytes per row of one part in LDS (padded: rows fall in different banks)
    constexpr int PartB = kStRows * RowB;
    constexpr int BufB = 3 * PartB;
    extern __shared__ __attribute__((aligned(16))) unsigned char st_smem[];
    unsigned char *Xb = st_smem;                                          // [4][BufB]
    float2 *red = reinterpret_cast<float2 *>(st_smem + 4 * BufB);         // [2][8][32] (value, index bits)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, g = lane >> 5;
    const int D4 = D >> 2;
    const f4 *__restrict__ X4 = reinterpret_cast<const f4 *>(X);
    const f4 *__restrict__ C4 = reinterpret_cast<const f4 *>(C);
    const long long t0 = blockIdx.x * tiles_per_block;
    const long long t1 = t0 + tiles_per_block < tiles ? t0 + tiles_per_block : tiles;
    const int n = (int)(t1 - t0);

    // this wave's centroids as A operands: lane (li, g) holds columns 16 s + 8 g .. + 7 of centroid cbase + li
    const int cbase = gbase + 32 * wave;
    u4 ca[NS][3];
    {
        const u4 *__restrict__ Cs16 = reinterpret_cast<const u4 *>(Cs);
        const size_t plane16 = (size_t)Kp * Dp / 8;
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int p = 0; p < 3; ++p) ca[s][p] = Cs16[p * plane16 + ((size_t)(cbase + li) * Dp + 16 * s + 8 * g) / 8];
    }
    float cnr[16];                         // |c|^2 of the centroid behind accumulator register r
#pragma unroll
    for (int r = 0; r < 16; ++r) cnr[r] = cn[cbase + 8 * (r >> 2) + 4 * g + (r & 3)];

    // loader role: row lr of the tile, columns 8 seg .. + 7
    const int lr = tid >> 4, seg = tid & 15;
    const bool loads = seg < Dp / 8;
    f4 mr0 = {0.0f, 0.0f, 0.0f, 0.0f}, mr1 = mr0;      // the common shift of this thread's columns
    if (loads) {
        const f4 *__restrict__ M4 = reinterpret_cast<const f4 *>(mean);
        if (2 * seg < D4) mr0 = M4[2 * seg];
        if (2 * seg + 1 < D4) mr1 = M4[2 * seg + 1];
    }
    // distance role: row 4 wave + rl of the tile, columns 8 part .. + 7
    const int rl = lane >> 4, part = lane & 15;
    const int erow = 4 * wave + rl;

#define SLAQ_ST_LOAD(T)                                                                      \
    {                                                                                        \
        const long long row_ = (T) * kStRows + lr;                                           \
        xr0 = f4{0.0f, 0.0f, 0.0f, 0.0f}; xr1 = xr0;                                         \
        if (loads && row_ < N) {                                                             \
            if (2 * seg < D4) xr0 = __builtin_nontemporal_load(X4 + row_ * D4 + 2 * seg);    \
            if (2 * seg + 1 < D4) xr1 = __builtin_nontemporal_load(X4 + row_ * D4 + 2 * seg + 1); \
        }                                                                                    \
    }
#define SLAQ_ST_STASH(B)                                                                     \
    if (loads) {                                                                             \
        /* the shift is taken off here, where the loaded values are first needed (columns    \
           past D hold zero in both) */                                                      \
        const f4 xs0_ = xr0 - mr0, xs1_ = xr1 - mr1;                                         \
        const float x_[8] = {xs0_.x, xs0_.y, xs0_.z, xs0_.w, xs1_.x, xs1_.y, xs1_.z, xs1_.w}; \
        u4 wh_, wm_, wl_;                                                                    \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                      \
            unsigned h0, m0, l0, h1, m1, l1;                                                 \
            split3(x_[2 * e], h0, m0, l0);                                                   \
            split3(x_[2 * e + 1], h1, m1, l1);                                               \
            wh_[e] = (h0 >> 16) | h1; wm_[e] = (m0 >> 16) | m1; wl_[e] = (l0 >> 16) | l1;    \
        }                                                                                    \
        unsigned char *dst_ = Xb + (B) * BufB + lr * RowB + seg * 16;                        \
        *reinterpret_cast<u4 *>(dst_) = wh_;                                                 \
        *reinterpret_cast<u4 *>(dst_ + PartB) = wm_;                                         \
        *reinterpret_cast<u4 *>(dst_ + 2 * PartB) = wl_;                                     \
    }

    // The four pieces of work of one trip i (between two barriers):
    //   NEAREST(j): rows of tile j: minimum over the 8 waves' results (ascending index, strict),
    //               merge with earlier centroid groups, start loading the chosen centroid
    //   MATRIX(i) : tile i on the matrix cores, this wave's nearest centroid per row to LDS
    //   DISTANCE(j): squared distance of tile j's rows to their centroids, from the definition
    //   FEED(i)   : tile i + 1 into LDS, tile i + 2 from HBM
    // None of them depends on another one of the same trip, so the two waves that share a SIMD
    // run them in different orders: while one is on the matrix cores the other does vector work.
#define SLAQ_ST_NEAREST(J)                                                                   \
    if ((J) >= 0 && (J) < n) {                                                               \
        const long long prow_ = (t0 + (J)) * kStRows + erow;                                 \
        const float2 *rp_ = red + ((J) & 1) * (kStWaves * kStRows) + erow;                   \
        float v_ = rp_[0].x; int k_ = __float_as_int(rp_[0].y);                              \
        _Pragma("unroll") for (int w_ = 1; w_ < kStWaves; ++w_) {                            \
            const float2 o_ = rp_[w_ * kStRows];                                             \
            if (o_.x < v_) { v_ = o_.x; k_ = __float_as_int(o_.y); }                         \
        }                                                                                    \
        if (!first && prow_ < N) {          /* earlier groups hold lower indices: they win ties */ \
            const float pv_ = bestv[prow_];                                                  \
            if (pv_ <= v_) { v_ = pv_; k_ = assign[prow_]; }                                 \
        }                                                                                    \
        ek = k_;                                                                             \
        if (!last) {                                                                         \
            if (part == 0 && prow_ < N) { bestv[prow_] = v_; assign[prow_] = k_; }           \
        } else {                                                                             \
            ec0 = f4{0.0f, 0.0f, 0.0f, 0.0f}; ec1 = ec0;                                     \
            if (2 * part < D4) ec0 = C4[(size_t)k_ * D4 + 2 * part];                         \
            if (2 * part + 1 < D4) ec1 = C4[(size_t)k_ * D4 + 2 * part + 1];                 \
        }                                                                                    \
    }
#define SLAQ_ST_MATRIX(I)                                                                    \
    if ((I) < n) {                                                                           \
        floatx16 accA = {0}, accB = {0};                                                     \
        const unsigned char *bp_ = Xb + ((I) & 3) * BufB + li * RowB + g * 16;               \
        _Pragma("unroll") for (int s_ = 0; s_ < NS; ++s_) {                                  \
            const u4 xh_ = *reinterpret_cast<const u4 *>(bp_ + s_ * 32);                     \
            const u4 xm_ = *reinterpret_cast<const u4 *>(bp_ + PartB + s_ * 32);             \
            const u4 xl_ = *reinterpret_cast<const u4 *>(bp_ + 2 * PartB + s_ * 32);         \
            accA = km_mfma_bf16(ca[s_][0], xl_, accA);                                       \
            accB = km_mfma_bf16(ca[s_][1], xm_, accB);                                       \
            accA = km_mfma_bf16(ca[s_][2], xh_, accA);                                       \
            accB = km_mfma_bf16(ca[s_][0], xm_, accB);                                       \
            accA = km_mfma_bf16(ca[s_][1], xh_, accA);                                       \
            accB = km_mfma_bf16(ca[s_][0], xh_, accB);                                       \
        }                                                                                    \
        /* registers in ascending centroid order, then the partner lane */                   \
        float v_ = std::numeric_limits<float>::infinity(); int k_ = cbase;                   \
        _Pragma("unroll") for (int r_ = 0; r_ < 16; ++r_) {                                  \
            const float val_ = __builtin_fmaf(-2.0f, accA[r_] + accB[r_], cnr[r_]);          \
            if (val_ < v_) { v_ = val_; k_ = cbase + 8 * (r_ >> 2) + 4 * g + (r_ & 3); }     \
        }                                                                                    \
        const float ov_ = __shfl_xor(v_, 32, 64);                                            \
        const int ok_ = __shfl_xor(k_, 32, 64);                                              \
        if (ov_ < v_ || (ov_ == v_ && ok_ < k_)) { v_ = ov_; k_ = ok_; }                     \
        if (g == 0) red[((I) & 1) * (kStWaves * kStRows) + wave * kStRows + li] = float2{v_, __int_as_float(k_)}; \
    }
#define SLAQ_ST_DISTANCE(J)                                                                  \
    if (last && (J) >= 0 && (J) < n) {                                                       \
        const long long prow_ = (t0 + (J)) * kStRows + erow;                                 \
        const unsigned char *xp_ = Xb + ((J) & 3) * BufB + erow * RowB + part * 16;          \
        u4 ph_ = {0, 0, 0, 0}, pm_ = ph_, pl_ = ph_;                                         \
        if (part < Dp / 8) {                                                                 \
            ph_ = *reinterpret_cast<const u4 *>(xp_);                                        \
            pm_ = *reinterpret_cast<const u4 *>(xp_ + PartB);                                \
            pl_ = *reinterpret_cast<const u4 *>(xp_ + 2 * PartB);                            \
        }                                                                                    \
        const float cc_[8] = {ec0.x, ec0.y, ec0.z, ec0.w, ec1.x, ec1.y, ec1.z, ec1.w};       \
        float d_ = 0.0f;                                                                     \
        _Pragma("unroll") for (int e_ = 0; e_ < 4; ++e_) {                                   \
            const float xa0_ = (__uint_as_float(ph_[e_] << 16) + __uint_as_float(pm_[e_] << 16)) + __uint_as_float(pl_[e_] << 16); \
            const float xa1_ = (__uint_as_float(ph_[e_] & 0xFFFF0000u) + __uint_as_float(pm_[e_] & 0xFFFF0000u)) + \
                               __uint_as_float(pl_[e_] & 0xFFFF0000u);                       \
            const float u0_ = xa0_ - cc_[2 * e_], u1_ = xa1_ - cc_[2 * e_ + 1];              \
            d_ = __builtin_fmaf(u0_, u0_, d_); d_ = __builtin_fmaf(u1_, u1_, d_);            \
        }                                                                                    \
        _Pragma("unroll") for (int o_ = 1; o_ <= 8; o_ <<= 1) d_ += __shfl_xor(d_, o_, 64);  \
        if (part == 0 && prow_ < N) { assign[prow_] = ek; dsum += d_; }                      \
    }
#define SLAQ_ST_FEED(I)                                                                      \
    {                                                                                        \
        if ((I) + 1 < n) SLAQ_ST_STASH(((I) + 1) & 3)                                        \
        if ((I) + 2 < n) SLAQ_ST_LOAD(t0 + (I) + 2)                                          \
    }

    f4 xr0, xr1;
    float dsum = 0.0f;                     // this lane's rows, in tile order (distance role, part 0)
    if (n > 0) {
        SLAQ_ST_LOAD(t0)
        SLAQ_ST_STASH(0)
        if (n > 1) SLAQ_ST_LOAD(t0 + 1)
    }
    __syncthreads();

    int ek = 0; f4 ec0 = {0.0f, 0.0f, 0.0f, 0.0f}, ec1 = ec0;      // distance role: chosen centroid and its columns
    // In trip i the buffers of tiles i - 2, i - 1 and i are read and that of tile i + 1 is
    // written: four buffers.  The results of tile i (red) are written in trip i and read in i + 1.
    if (wave < kStWaves / 2) {
        for (int i = 0; i <= n + 1; ++i) {
            SLAQ_ST_DISTANCE(i - 2)        // its centroid was requested in the previous trip
            SLAQ_ST_FEED(i)
            SLAQ_ST_NEAREST(i - 1)
            SLAQ_ST_MATRIX(i)
            __syncthreads();
        }
    } else {
        for (int i = 0; i <= n + 1; ++i) {
            SLAQ_ST_NEAREST(i - 1)
            SLAQ_ST_MATRIX(i)              // hides the latency of the centroid request
            SLAQ_ST_DISTANCE(i - 1)
            SLAQ_ST_FEED(i)
            __syncthreads();
        }
    }
#undef SLAQ_ST_NEAREST
#undef SLAQ_ST_MATRIX
#undef SLAQ_ST_DISTANCE
#undef SLAQ_ST_FEED
#undef SLAQ_ST_LOAD
#undef SLAQ_ST_STASH
    if (last) {
        // the wave's four row lanes (part 0 of each quarter), fixed order
        const float s0 = __shfl(dsum, 0, 64), s1 = __shfl(dsum, 16, 64), s2 = __shfl(dsum, 32, 64), s3 = __shfl(dsum, 48, 64);
        if (lane == 0) lossW[blockIdx.x * kStWaves + wave] = ((s0 + s1) + s2) + s3;
    }
}

// One wave = (row split p, slab of 64 columns, owner group w).  Cluster k belongs to group k % G
// and is that group's local cluster k / G (< 32); a wave keeps the sums of its 32 local clusters
// for its column in registers and reads from X only the rows assigned to them, in row order, so
// every sum has a fixed order and no two waves add into the same place.  The cluster index of a
// row is wave-uniform, hence the register array is indexed by a scalar.
typedef float floatx32 __attribute__((ext_vector_type(32)));
constexpr int kAccJ = 8;                   // rows gathered per round

// LOSS: the pass also adds sum_j (x_ij - c_kj)^2 with the entering centroid of the row's cluster
// (read through the cache, next to the row itself) and writes one partial per wave; used when the
// assignment kernel does not produce the loss.
template <bool LOSS>
__global__ __launch_bounds__(256) void kmeans_accumulate_kernel(
    const float *__restrict__ X, const float *__restrict__ C, const int *__restrict__ assign, long long N, int D,
    int K, int G, int nslab, long long rows_per_split, long long total_waves, float *__restrict__ part,
    int *__restrict__ cntP, float *__restrict__ lossP) {
    const int lane = threadIdx.x & 63;
    const long long wg = blockIdx.x * 4LL + (threadIdx.x >> 6);
    if (wg >= total_waves) return;
    const int w = (int)(wg % G);
    const long long t = wg / G;
    const int slab = (int)(t % nslab);
    const long long p = t / nslab;
    const int col = slab * 64 + lane;
    const bool active = col < D;
    const long long rb = p * rows_per_split;
    const long long re = rb + rows_per_split < N ? rb + rows_per_split : N;
    const float *__restrict__ xc = X + (active ? col : 0);

    floatx32 acc = {0};
    const float *__restrict__ cc = C + (active ? col : 0);
    float dsum = 0.0f;                     // LOSS: this lane's column, rows in order
    int size = 0;                          // lane l counts the rows of local cluster l
    for (long long r = rb; r < re; r += 64) {
        const long long row = r + lane;
        const int av = row < re ? assign[row] : -1;
        const int local = av / G;
        unsigned long long mask = __ballot(av >= 0 && av - local * G == w);
        while (mask) {
            float v[kAccJ], c[kAccJ]; int a[kAccJ];
#pragma unroll
            for (int j = 0; j < kAccJ; ++j) {
                a[j] = -1; v[j] = 0.0f; c[j] = 0.0f;
                if (mask) {
                    const int u = __builtin_ctzll(mask);
                    mask &= mask - 1;
                    a[j] = __builtin_amdgcn_readlane(local, u);
                    v[j] = __builtin_nontemporal_load(xc + (r + u) * D);
                    if (LOSS) c[j] = cc[(size_t)(a[j] * G + w) * D];
                }
            }
#pragma unroll
            for (int j = 0; j < kAccJ; ++j)
                if (a[j] >= 0) {
                    acc[a[j]] += v[j];
                    if (LOSS) {
                        const float t_ = v[j] - c[j];
                        dsum = __builtin_fmaf(t_, t_, dsum);
                    }
                    size += lane == a[j] ? 1 : 0;
                }
        }
    }
#pragma unroll
    for (int l = 0; l < 32; ++l) {
        const int k = l * G + w;
        if (k < K && active) part[((size_t)p * K + k) * D + col] = acc[l];
    }
    if (slab == 0 && lane < 32 && lane * G + w < K) cntP[(size_t)p * K + lane * G + w] = size;
    if (LOSS) {
        if (!active) dsum = 0.0f;
        for (int o = 32; o >= 1; o >>= 1) dsum += __shfl_xor(dsum, o, 64);
        if (lane == 0) lossP[wg] = dsum;
    }
}

__global__ __launch_bounds__(256) void kmeans_finalize_kernel(
    const float *__restrict__ part, const int *__restrict__ cntP, const float *__restrict__ lossP, long long T,
    int P, long long N, int D, int K, float *__restrict__ C, int *__restrict__ counts, float *__restrict__ loss_out) {
    __shared__ int redi[256];
    __shared__ double redd[256];
    // block (k, slab of 16 columns); thread = (split lane pl of 16, column dc of 16)
    const int k = blockIdx.x, tid = threadIdx.x;
    int n = 0;
    for (int p = tid; p < P; p += 256) n += cntP[(size_t)p * K + k];
    redi[tid] = n;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if (tid < s) redi[tid] += redi[tid + s];
        __syncthreads();
    }
    const int size = redi[0];
    if (tid == 0 && blockIdx.y == 0) counts[k] = size;
    const int pl = tid >> 4, dc = tid & 15;
    const int d = blockIdx.y * 16 + dc;
    {
        // splits pl, pl + 16, ... in order, then the sixteen lanes in order: a fixed sequence
        double tot = 0.0;
        if (d < D) {
            const float *__restrict__ pp = part + (size_t)k * D + d;
            const size_t stride = (size_t)K * D;
            int p = pl;
            for (; p + 16 * 7 < P; p += 16 * 8) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = pp[(size_t)(p + 16 * u) * stride];
#pragma unroll
                for (int u = 0; u < 8; ++u) tot += (double)v[u];
            }
            for (; p < P; p += 16) tot += (double)pp[(size_t)p * stride];
        }
        redd[tid] = tot;
        __syncthreads();
        if (pl == 0 && d < D) {
            for (int q = 1; q < 16; ++q) tot += redd[16 * q + dc];
            if (size > 0) C[(size_t)k * D + d] = (float)(tot / (double)size);
        }
        __syncthreads();
    }
    if (k == 0 && blockIdx.y == 0) {
        // loss: thread t adds a contiguous run of the tile partials, then a fixed tree
        double s = 0.0;
        for (long long t = T * tid / 256; t < T * (tid + 1) / 256; ++t) s += (double)lossP[t];
        redd[tid] = s;
        __syncthreads();
        for (int h = 128; h >= 1; h >>= 1) {
            if (tid < h) redd[tid] += redd[tid + h];
            __syncthreads();
        }
        if (tid == 0) *loss_out = (float)(redd[0] / (double)N);
    }
}

template <int TR>
static hipError_t launch_assign(const KmArgs &a, hipStream_t st) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&kmeans_assign_kernel<TR>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.s.lds_assign);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kmeans_assign_kernel<TR>, dim3((unsigned)a.s.T), dim3(TR * 2), a.s.lds_assign, st, a.X, a.Cc,
                       a.mean, a.cn, a.N, a.D, a.K, a.s.Dp, a.s.Kp, a.assign, a.lossP);
    return hipGetLastError();
}

hipError_t launch_kmeans_iteration(const KmArgs &a, int k, hipEvent_t *ev, hipStream_t st) {
    hipError_t e;
    int dev = 0, lds_max = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev)) != hipSuccess) return e;
    if ((size_t)lds_max < a.s.lds_assign) return hipErrorInvalidValue;

    if (k == 0) {                          // the shift depends on X only: once per call
        hipLaunchKernelGGL(kmeans_mean_kernel, dim3((unsigned)((a.D + 63) / 64)), dim3(64 * kKmMeanWaves), 0, st, a.X, a.N, a.D,
                           a.mean);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kmeans_center_kernel, dim3((unsigned)((a.s.Kp + 3) / 4)), dim3(256), 0, st, a.C, a.mean, a.D,
                       a.K, a.s.Kp, a.Cc, a.cn);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (a.s.split) {
        const long long n = (long long)a.s.Kp * a.s.Dp;
        hipLaunchKernelGGL(kmeans_split_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a.Cc, a.D, a.K,
                           a.s.Kp, a.s.Dp, a.Cs);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (ev && (e = hipEventRecord(ev[0], st)) != hipSuccess) return e;
    if (a.s.small) {
        const dim3 grid((unsigned)a.s.T), block(kKmSmallRows);
        switch ((a.K + 7) / 8) {
        case 1: hipLaunchKernelGGL(kmeans_assign_small_kernel<1>, grid, block, 0, st, a.X, a.Cc, a.mean, a.cn, a.N, a.D, a.K, a.assign); break;
        case 2: hipLaunchKernelGGL(kmeans_assign_small_kernel<2>, grid, block, 0, st, a.X, a.Cc, a.mean, a.cn, a.N, a.D, a.K, a.assign); break;
        case 3: hipLaunchKernelGGL(kmeans_assign_small_kernel<3>, grid, block, 0, st, a.X, a.Cc, a.mean, a.cn, a.N, a.D, a.K, a.assign); break;
        case 4: hipLaunchKernelGGL(kmeans_assign_small_kernel<4>, grid, block, 0, st, a.X, a.Cc, a.mean, a.cn, a.N, a.D, a.K, a.assign); break;
        case 5: hipLaunchKernelGGL(kmeans_assign_small_kernel<5>, grid, block, 0, st, a.X, a.Cc, a.mean, a.cn, a.N, a.D, a.K, a.assign); break;
        case 6: hipLaunchKernelGGL(kmeans_assign_small_kernel<6>, grid, block, 0, st, a.X, a.Cc, a.mean, a.cn, a.N, a.D, a.K, a.assign); break;
        case 7: hipLaunchKernelGGL(kmeans_assign_small_kernel<7>, grid, block, 0, st, a.X, a.Cc, a.mean, a.cn, a.N, a.D, a.K, a.assign); break;
        default: hipLaunchKernelGGL(kmeans_assign_small_kernel<8>, grid, block, 0, st, a.X, a.Cc, a.mean, a.cn, a.N, a.D, a.K, a.assign); break;
        }
        e = hipGetLastError();
    } else if (a.s.split) {
        const size_t lds = (size_t)4 * 3 * kStRows * (2 * a.s.Dp + 16) + 2 * kStWaves * kStRows * sizeof(float2);
        const void *fn = a.s.Dp == 64 ? reinterpret_cast<const void *>(&kmeans_assign_stream_kernel<1>)
                                      : reinterpret_cast<const void *>(&kmeans_assign_stream_kernel<2>);
        if ((e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)) != hipSuccess) return e;
        const int groups = a.s.Kp / kStGroup;
        for (int gi = 0; gi < groups && e == hipSuccess; ++gi) {
            const int first = gi == 0, last = gi == groups - 1;
            if (a.s.Dp == 64)
                hipLaunchKernelGGL(kmeans_assign_stream_kernel<1>, dim3((unsigned)a.s.stream_blocks), dim3(512), lds, st,
                                   a.X, a.Cc, a.mean, a.Cs, a.cn, a.N, a.D, a.s.Kp, gi * kStGroup, first, last, a.s.T,
                                   a.s.tiles_per_block, a.assign, a.bestv, a.lossP);
            else
                hipLaunchKernelGGL(kmeans_assign_stream_kernel<2>, dim3((unsigned)a.s.stream_blocks), dim3(512), lds, st,
                                   a.X, a.Cc, a.mean, a.Cs, a.cn, a.N, a.D, a.s.Kp, gi * kStGroup, first, last, a.s.T,
                                   a.s.tiles_per_block, a.assign, a.bestv, a.lossP);
            e = hipGetLastError();
        }
    } else if (a.s.TR == 128) e = launch_assign<128>(a, st);
    else if (a.s.TR == 64) e = launch_assign<64>(a, st);
    else e = launch_assign<32>(a, st);
    if (e != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[1], st)) != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[2], st)) != hipSuccess) return e;
    const long long waves = (long long)a.s.P * a.s.nslab * a.s.G;
    if (a.s.small)
        hipLaunchKernelGGL(kmeans_accumulate_kernel<true>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, a.X, a.C,
                           a.assign, a.N, a.D, a.K, a.s.G, a.s.nslab, a.s.rows_per_split, waves, a.part, a.cntP, a.lossP);
    else
        hipLaunchKernelGGL(kmeans_accumulate_kernel<false>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, a.X, a.C,
                           a.assign, a.N, a.D, a.K, a.s.G, a.s.nslab, a.s.rows_per_split, waves, a.part, a.cntP, a.lossP);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[3], st)) != hipSuccess) return e;
    hipLaunchKernelGGL(kmeans_finalize_kernel, dim3((unsigned)a.K, (unsigned)((a.D + 15) / 16)), dim3(256), 0, st, a.part, a.cntP, a.lossP, a.s.lossN,
                       a.s.P, a.N, a.D, a.K, a.C, a.counts, a.loss_out + k);
    return hipGetLastError();
}

}  // namespace slaqglm
