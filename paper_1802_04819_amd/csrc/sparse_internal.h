// Row-panelled column layout of the sparse iteration (glm_sparse.hip, driven from glm_api_jobs.hip).
#pragma once

#include "glm_internal.h"

namespace slaqglm {

constexpr long long kSparsePanelRows = 512 * 1024;   // residuals of one panel: 2 MB, well inside one L2
constexpr int kSparseMaxPanels = 64;
constexpr int kScanBlock = 4096;                      // items per block of the prefix sum

// The column pass gathers from the residual vector r [N].  Beyond a few MB r no longer stays in
// L2 and every gather of 4 bytes pulls a whole line from memory.  So the column layout is
// rebuilt once, in the workspace, ordered by row panel first: panel p holds, column by column,
// the entries whose row lies in [p R, (p + 1) R).  The column pass then is the same segmented sum
// over P * D segments, and while the entries of panel p stream by, only r [p R, (p + 1) R) is hot.
struct SparsePanels {
    int P;               // 1: the caller's column layout is used as it is
    long long R;         // rows per panel
    long long *pp;       // [(P + 1) * D] first entry of each column with row >= p R
    long long *ptr2;     // [P * D + 1]   segment starts of the panelled layout
    long long *bsum;     // [blocks + 1]  block totals of the prefix sum
    int *idx2;           // [nnz] row of every entry, panelled order
    float *val2;         // [nnz]
    int *seg0;           // [nch + 1] segment holding each chunk's first entry
    float *gs2;          // [P * D] column sums per panel
    int *flag;           // [1] set if some column's rows are not in ascending order
};
int sparse_panel_count(long long N, long long D);
hipError_t launch_sparse_sorted_check(const SparseArgs &a, const SparsePanels &pn, hipStream_t st);
hipError_t launch_sparse_panel_build(const SparseArgs &a, const SparsePanels &pn, hipStream_t st);
hipError_t launch_sparse_iteration_panels(const SparseArgs &a, const SparsePanels &pn, int k, hipEvent_t *ev,
                                          hipStream_t st);

// ---- column layout built by the library (glm_sparse_csc.hip), for callers that give CSR only ----
struct SparseCsc {
    long long *col_ptr;              // [D + 1]
    int *row_idx;                    // [nnz]
    float *col_val;                  // [nnz]
    int *keys[2];                    // [nnz] each: column indices, the sort's two buffers
    unsigned long long *vals[2];     // [nnz] each: (row << 32) | value bits
    void *temp;                      // scratch of the sort
    size_t temp_bytes;
};
size_t sparse_csc_temp_bytes(long long nnz);
hipError_t launch_sparse_csc_build(const SparseArgs &a, const SparseCsc &c, hipStream_t st);

// ---- scatter into LDS with fixed-point sums (glm_sparse_fx.hip) --------------------------------
constexpr int kFxPanel = 16384;              // outputs per panel: their 64-bit sums fill 128 KB of LDS
constexpr int kFxPanelBits = 14;
constexpr int kFxMaxPanels = 1024;           // bins of the split that builds the layout
constexpr int kFxWindowBits = 18;            // a window of the gathered vector: what 32 - kFxPanelBits bits address
constexpr int kFxMaxWindows = 64;
constexpr int kFxRun = 4096;                 // entries of one (panel, window) run are padded to a multiple of this
constexpr long long kFxMinEntries = 1LL << 22;
constexpr int kFxBlocks = 256;               // at most one block per compute unit: the sums of a panel fill its LDS
// device scalars of the path (unsigned [kFxSlots])
enum : int { kFxSlotMaxW = 0, kFxSlotMaxR = 1, kFxSlotMaxVal = 2, kFxSlotERow = 3, kFxSlotECol = 4, kFxSlotLenRow = 5,
             kFxSlotLenCol = 6, kFxSlots = 8 };
struct FxPass {
    int on;                  // this pass takes the path
    int P;                   // panels of the output vector
    int W;                   // windows of the gathered vector
    long long span;          // consecutive entries of the padded stream per block (a multiple of kFxRun)
    int blocks;              // blocks of the pass: block k streams entries [k span, (k + 1) span)
    long long slices;        // blocks + P: block k writes its sums for panel p to slice k + p
    long long out_len;       // N for the row pass, D for the column pass
    long long gather_len;    // D for the row pass, N for the column pass
    long long ntiles;        // tiles of the split (an upper bound: no tile crosses a window of the source)
    long long cap;           // entries the padded stream can hold: a multiple of kFxRun
    unsigned *ent;           // [cap] output index inside the panel | (gathered index - start of its window) << 14
    float *val;              // [cap]; the entries of one panel and one window form a run, padded with zero
                             //   entries to a multiple of kFxRun: a group of kFxRun entries has one window
    int *tbase;              // [cap / kFxRun] first gathered index of the window of each such group
    long long *pstart;       // [P + 1] first entry of each panel
    long long *shift;        // [P * W] how far the entries of a run move up for the padding before them
    long long *rstart;       // [P * W] first entry of each run
    long long *rlen;         // [P * W] entries of each run before padding
    long long *wsrc;         // [W + 1] first source entry of each window
    long long *tfirst;       // [W + 1] first tile of each window
    long long *part;         // [slices, kFxPanel] fixed-point partial sums
};
struct SparseFx {
    FxPass row, col;
    unsigned *slots;         // [kFxSlots]
    long long *cnt;          // [max(P) * ntiles + 1] split counters
    long long *bsum;         // block totals of their prefix sum
};
void sparse_fx_plan(long long N, long long D, long long nnz, FxPass *row, FxPass *col);
hipError_t launch_sparse_fx_build(const SparseArgs &a, const SparseFx &fx, hipStream_t st);
hipError_t launch_sparse_fx_begin(const SparseArgs &a, const SparseFx &fx, hipStream_t st);
hipError_t launch_sparse_fx_pass(const SparseFx &fx, bool row, const float *vec, long long vec_len, long long nnz,
                                 float *out, hipStream_t st);
hipError_t launch_sparse_iteration_any(const SparseArgs &a, const SparsePanels &pn, const SparseFx &fx, int k,
                                       hipEvent_t *ev, hipStream_t st);

}  // namespace slaqglm
