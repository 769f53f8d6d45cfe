// Host-side declarations shared by the kernel files and the C ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/seer.h"

namespace seer {

constexpr int kBmMaxRows = 2048;  // most rows one CSR,BM workgroup owns (8 per lane, bounds in registers)
constexpr int kAutoBmMaxRows = 1024;   // ... inside the combined kernel (4 per lane: keeps it at eight waves per SIMD)
constexpr int kBmChunk = 2048;    // products staged in LDS per CSR,BM pass (4096 is the other choice)
constexpr int kMpIptSmall = 7;    // merge items per thread, small problems (tile = 1792 items)
constexpr int kMpIptLarge = 15;   // merge items per thread, large problems (tile = 3840 items)

struct SpmvArgs {
    int rows, cols, nnz;
    const int *rp, *ci;
    const float *va, *x;
    float *y;
    int remap;  // 1: tiles laid out contiguously per XCD
    int nt;     // 1: matrix streams are loaded with the non-temporal hint (keeps x in L2)
};

bool tm_short_rows(int rows, int nnz);
int tm_rows_per_lane(int rows, int nnz);
uint32_t tm_num_tiles(int rows, int nnz);
void launch_tm(const SpmvArgs &a, hipStream_t st);
void launch_wm(const SpmvArgs &a, int lanes_per_row, hipStream_t st);
void launch_bm(const SpmvArgs &a, int rows_per_block, int chunk, bool vec, hipStream_t st);

// merge path: ipt is kMpIptSmall or kMpIptLarge
uint32_t mp_num_tiles(int rows, int nnz, int ipt);
size_t mp_workspace_bytes(int rows, int nnz, int ipt);
void launch_mp(const SpmvArgs &a, int ipt, bool vec, void *workspace, hipStream_t st);

// work oriented (nonzero split); shares the carry arrays' layout and the fix-up with merge path
uint32_t wo_num_tiles(int rows, int nnz);
void launch_wo(const SpmvArgs &a, bool vec, void *workspace, hipStream_t st);
size_t carry_workspace_bytes(uint32_t n_tiles);
void launch_carry_fixup(int rows, uint32_t n_tiles, const int *carry_row, const float *carry_val, float *y,
                        hipStream_t st);

// adaptive (row blocks found by a preprocessing pass).  plan_mem: adaptive_plan_bytes();
// carry_ws: carry_workspace_bytes(adaptive_num_tiles()) or null when the plan has no split row
uint32_t adaptive_num_tiles(int rows, int nnz);
size_t adaptive_plan_bytes(int rows, int nnz);
int *adaptive_split_flag(void *plan_mem, int rows, int nnz);
void launch_adaptive_plan(int rows, int nnz, const int *rp, void *plan_mem, bool want_flag, hipStream_t st);
void launch_adaptive(const SpmvArgs &a, bool vec, const void *plan_mem, void *carry_ws, hipStream_t st);

// ELL,TM: plan_mem holds the ELL columns, then the ELL values (ell_plan_bytes())
uint32_t ell_rows_pad(int rows);
size_t ell_plan_bytes(int rows, int width);
void launch_ell_convert(int rows, int width, const int *rp, const int *ci, const float *va, void *plan_mem,
                        hipStream_t st);
void launch_ell(const SpmvArgs &a, int width, const void *plan_mem, hipStream_t st);

// COO,WM: plan_mem holds the row index of every nonzero; carry_ws: carry_workspace_bytes(coo_num_intervals())
uint32_t coo_num_intervals(int rows, int nnz);
size_t coo_plan_bytes(int rows, int nnz);
void launch_coo_convert(int rows, const int *rp, void *plan_mem, hipStream_t st);
void launch_coo(const SpmvArgs &a, bool runs /* lane-owned runs of triples (the default form) */, const void *plan_mem,
                void *carry_ws, hipStream_t st);

// CSR,S: plan_mem holds the kept virtual rows' offsets, each row's list of pieces, the slabbed
// col_idx and values, then the preprocessing's scratch (slab_plan_bytes());
// workspace: slab_workspace_bytes() (one partial per kept virtual row, then CSR,WO's carries)
constexpr int kSlabShift = 19;              // a slab of x: 2^19 columns = 2 MiB, half of one XCD's L2
uint32_t slab_count(int rows, int cols, int shift);     // 0: the form does not apply (one slab, or too many virtual rows)
size_t slab_plan_bytes(int rows, int cols, int nnz, int shift);
size_t slab_workspace_bytes(uint32_t n_kept, int nnz);
int *slab_flag(void *plan_mem, int rows, int cols, int nnz, int shift);
const uint32_t *slab_kept_count(const void *plan_mem, int rows, int cols, int nnz, int shift);
void launch_slab_count(int rows, int cols, int nnz, int shift, const int *rp, const int *ci, void *plan_mem, hipStream_t st);
void launch_slab_fill(int rows, int cols, int nnz, int shift, uint32_t n_kept, const int *rp, const int *ci, const float *va,
                      void *plan_mem, hipStream_t st);
void launch_slab(const SpmvArgs &a, uint32_t n_slabs, uint32_t n_kept, const void *plan_mem, void *workspace, hipStream_t st);

// feature reduction
struct FeatureRaw {           // written by the device into pinned host memory
    int32_t max_len, min_len;
    int32_t first, last;      // row_ptr[0], row_ptr[rows]
    uint64_t sum_sq, empty;
    uint64_t seq;             // call counter echoed back (host checks it moved)
};
size_t features_workspace_bytes(int rows);
void launch_features(int rows, const int *rp, void *workspace, FeatureRaw *mailbox_dev,
                     uint64_t seq, hipStream_t st);

// CSR,BM: when a block owns fewer rows than it has lanes, every 2^shift-th lane owns one
inline int bm_own_shift(int rows_per_block)
{
    int shift = 0;
    while ((rows_per_block << (shift + 1)) <= 256) ++shift;
    return shift;
}

// ---- asynchronous path: selection on the device, one combined SpMV kernel
constexpr int kAutoMaxNodes = 127;          // a depth-6 binary tree; fits the 4 KB kernel-argument block
struct AutoTree {                           // passed to the kernel by value
    int32_t n_nodes, pad;
    seer_node nodes[kAutoMaxNodes];
};
// A tree of depth <= 6 laid out as a complete binary tree (slot i has children 2i + 1 and
// 2i + 2): one wave can then load every node at once, evaluate all comparisons in parallel
// and find the leaf with bit operations, instead of one dependent load per level.
constexpr int kHeapInternal = 63;           // slots 0..62 can be internal nodes, 63..126 are leaves
struct AutoHeap {                           // passed to the kernel by value (896 bytes)
    int32_t feature[64];                    // -1: the slot is a leaf (or not reachable)
    double threshold[64];
    int8_t klass[128];                      // kernel id of every slot that is a leaf
};
bool flatten_tree(const seer_tree *tree, AutoHeap *heap);   // false: deeper than 6 levels of comparisons

struct AutoSel {                            // what the selection leaves in the workspace
    int32_t kernel_id, valid;               // valid: 1 gathered on the device; 2 decided on the host, no statistics
    int64_t rows, cols, nnz;
    int32_t max_len, min_len;
    uint64_t sum_sq, empty;
    float f[SEER_NUM_FEATURES];
};
struct AutoShape {                          // launch shapes, all from rows and nnz alone
    uint32_t tiles[SEER_NUM_DIRECT_KERNELS];
    int wm_lanes, bm_rows, bm_own_shift, mp_ipt;
    int tm_short;                           // CSR,TM fetches the first eight entries of a row at once (mean row length <= 8)
    int tm_pair;                            // ... and takes two rows per lane (tiles of 512 rows)
    int tm_remap;                           // CSR,TM's tile order: 1 XCD-contiguous, 0 round-robin
    uint32_t reachable;                     // bit k: the tree can answer kernel k given rows, cols and nnz (never 0)
};
constexpr size_t kAutoSelOffset = 32768;    // after the 1024 feature partials of 32 bytes
constexpr size_t kAutoCarryOffset = 32768 + 256;
size_t auto_workspace_bytes(int rows, int nnz);
constexpr int kAutoFusedRows = 8192;        // up to here every workgroup gathers and selects for itself, no first pass
constexpr int kAutoFusedGrid = 1024;        // the product's launch selects for itself up to this many workgroups ...
constexpr int kAutoFusedMaxRows = 0;        // ... and, whatever its grid, up to this many rows (off: measured slower; the first pass
                                            // of at most kAutoFusedParts workgroups is the slower way to read row_ptr)
constexpr uint32_t kAutoFusedParts = 64;    // partials the first pass leaves for it (one per lane of the folding wave)
constexpr uint32_t kAutoWmGrid = 4096;      // combined kernel: CSR,WM loops beyond max(this, the other schedules' grids)
struct AutoPolicy {                         // when the selection runs inside the product's launch
    int fused_rows, fused_grid, fused_max_rows;
    int select_wave;                        // 1: the selection launch is a single wave (0: a workgroup of 1024 lanes)
    uint32_t part_rows;                     // rows per workgroup of the first pass (0: the default)
};
// heap: the flattened tree, or null if it is too deep (then the node array is walked).
// decided: null, or the record of a choice the host could make alone (shape.reachable has
// one bit): nothing is gathered then.
void launch_auto(const SpmvArgs &a, const AutoTree &tree, const AutoHeap *heap, const AutoShape &shape, bool vec,
                 const AutoPolicy &policy, const AutoSel *decided, void *workspace, hipStream_t st);

void launch_csr_check(int rows, int cols, int nnz, const int *rp, const int *ci, void *counts, hipStream_t st);
void launch_stream_copy(void *dst, const void *src, size_t n_words, hipStream_t st);
void launch_gather_sum(const int *idx, const float *val, size_t n, const float *x, void *out64, hipStream_t st);
void launch_stream_sum(const void *src, size_t n_words, void *out64, hipStream_t st);

} // namespace seer
