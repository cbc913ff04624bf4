// Internal declarations of the K-Means iteration (kmeans.hip, driven from glm_api.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace slaqglm {

constexpr int kKmMaxD = 1024;           // the X tile of the assignment kernel must fit in LDS
constexpr int kKmMaxK = 1024;           // 32 owner groups of 32 clusters in the accumulation pass
constexpr int kKmSplitMaxD = 128;       // up to here a row's split operands fit in a lane pair's registers
constexpr int kKmChunk = 64;            // centroids per matrix-core chunk
constexpr int kKmSmallK = 64;           // up to here the assignment may run on the vector units, a row per lane
constexpr int kKmSmallWork = 4096;      // ... beyond 32 centroids only while K * D stays below this
constexpr int kKmSmallRows = 256;       // rows per block of that kernel

// Shapes derived from (N, D, K) alone, so that every call on the same problem runs the same
// launches and adds in the same order.
struct KmShape {
    bool small;          // few centroids: assignment on the vector units (a matrix tile would be mostly padding)
    bool split;          // otherwise, D <= 128: assignment with three-way bfloat16 operands
    int TR;              // rows per assignment tile (128, 64 or 32)
    int Dp;              // D rounded up to a multiple of 64 (split) or 32
    long long T;         // assignment tiles
    int stream_blocks;   // split path: persistent blocks
    long long tiles_per_block;
    long long lossN;     // loss partials written by the assignment kernel
    int Kp;              // K rounded up to a multiple of 64 (256 on the split path)
    int nslab;           // accumulation slabs of 64 columns
    int G;               // owner groups of the accumulation pass: cluster k belongs to group k % G
    long long rows_per_split;
    int P;               // row splits of the accumulation kernel
    size_t lds_assign;
};
KmShape km_shape(long long N, int D, int K);

struct KmArgs {
    const float *X; float *C; int *assign; int *counts; float *loss_out;
    long long N; int D, K;
    float *mean;         // [D] common shift: column means of a sample of the rows, once per call
    float *Cc;           // [K, D] centroids minus the shift
    float *cn;           // [Kp] squared norms of the shifted centroids, +inf past K
    unsigned short *Cs;  // [3, Kp, Dp] bfloat16 parts of the shifted centroids (split path)
    float *lossP;        // [lossN] partial sums of the squared distances
    float *bestv;        // [N] best value so far (split path with more than 256 centroids)
    float *part;         // [P, K, D] per-split column sums
    int *cntP;           // [P, K]    per-split cluster sizes
    KmShape s;
};
hipError_t launch_kmeans_iteration(const KmArgs &a, int k, hipEvent_t *ev, hipStream_t st);

}  // namespace slaqglm
