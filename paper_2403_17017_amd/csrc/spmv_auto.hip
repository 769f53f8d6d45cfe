// The whole runtime flow of Sec. III-B -- gather features, evaluate the decision tree,
// run the chosen kernel -- as a few launches with no host round trip in between:
//
//   1. the feature reduction (one launch for a small matrix, two for a large one);
//      its finishing workgroup (features_select_kernel) derives the feature vector
//      on the device, walks the tree (handed over by value in the kernel arguments)
//      and leaves the chosen kernel id in device memory;
//   2. spmv_auto_kernel: one kernel that contains the five CSR schedules that need no
//      preprocessing; every workgroup reads the chosen id and runs that schedule's
//      body (the grid is sized for the schedule that needs the most workgroups, the
//      rest exit);
//   3. spmv_auto_fixup_kernel: the carry fix-up of merge path and of the nonzero
//      split; exits at once unless one of them was chosen.
// When the product's grid is small, steps 1 and 2 share a launch (or, for a small
// matrix, are one launch): see spmv_auto_fused_kernel.
//
// The host only enqueues; feature collection costs the reduction kernel itself
// instead of a launch, a wait and a second launch.  The sequence has no host-side
// dependency on device data, so it can be captured in a HIP graph.
//
// The derivation of the floating-point features repeats the host's, operation by
// operation (exact integers, correctly rounded int -> fp64 conversions, one fp64
// division, one rounding to fp32), so both give the same bits.
#include "../../include/seer.h"
#include "features_bodies.hiph"
#include "spmv_bodies.hiph"

namespace seer {

// Correctly rounded (nearest-even) conversion of a 128-bit unsigned integer: keep
// the top 64 bits, fold everything below into the lowest kept bit (sticky), convert
// (64 -> 53 bits rounds once, and the sticky bit makes that the rounding of the
// full number), scale back exactly.
__device__ __forceinline__ double u128_to_double(unsigned __int128 n)
{
    const uint64_t hi = (uint64_t)(n >> 64);
    if (hi == 0) return (double)(uint64_t)n;
    const int s = 64 - __clzll((long long)hi);            // 1..64
    uint64_t top = (uint64_t)(n >> s);
    const unsigned __int128 below = n - ((unsigned __int128)top << s);
    top |= (uint64_t)(below != 0);
    return ldexp((double)top, s);
}

__device__ __forceinline__ void derive_features_device(
    int64_t rows, int64_t cols, int64_t nnz, int64_t max_len, int64_t min_len, int64_t empty,
    uint64_t sum_sq, float *f)
{
    for (int i = 0; i < SEER_NUM_FEATURES; ++i) f[i] = 0.0f;
    f[SEER_F_COLS] = (float)(double)cols;
    f[SEER_F_ITERATIONS] = 1.0f;   // this path is the single product
    if (rows <= 0) return;
    const double R = (double)rows;
    const double mean = (double)nnz / R;
    const unsigned __int128 num = (unsigned __int128)(uint64_t)rows * (unsigned __int128)sum_sq -
                                  (unsigned __int128)(uint64_t)nnz * (unsigned __int128)(uint64_t)nnz;
    const double var = u128_to_double(num) / (double)((uint64_t)rows * (uint64_t)rows);
    f[SEER_F_ROWS] = (float)R;
    f[SEER_F_NNZ] = (float)(double)nnz;
    f[SEER_F_MEAN_LEN] = (float)mean;
    f[SEER_F_MAX_LEN] = (float)(double)max_len;
    f[SEER_F_MIN_LEN] = (float)(double)min_len;
    f[SEER_F_VAR_LEN] = (float)var;
    f[SEER_F_EMPTY_FRAC] = (float)((double)empty / R);
    if (cols > 0) {
        const double C = (double)cols;
        f[SEER_F_MEAN_DENSITY] = (float)(mean / C);
        f[SEER_F_MAX_DENSITY] = (float)((double)max_len / C);
        f[SEER_F_MIN_DENSITY] = (float)((double)min_len / C);
        f[SEER_F_VAR_DENSITY] = (float)(var / (C * C));
    }
}

// One lane's work once the workgroup holds the matrix's statistics in *s: derive the
// feature vector (into LDS, so that the tree can index it without forcing it into
// private scratch memory), walk the tree where it lies in the kernel arguments, and, if
// `sel` is given, leave the record that seer_spmv_auto_result reads.  Returns the kernel
// id.  (Sharing the derivation between the waves and staging the tree in LDS first was
// measured: it is slower by more than a microsecond, the bulk read of the 3 KB argument
// block costs more than the few nodes a walk touches.)
__device__ __forceinline__ int select_on_device(
    int rows, int cols, const int *__restrict__ rp, const FeatLds *s, float *s_f, const AutoTree &tree,
    AutoSel *__restrict__ sel)
{
    const int64_t nnz = (int64_t)rp[rows] - (int64_t)rp[0];
    derive_features_device(rows, cols, nnz, s->mx, s->mn, (int64_t)s->em, s->sq, s_f);
    int n = 0, k = SEER_CSR_MP;            // a malformed tree cannot get here (host checks); MP is the safe answer
    for (int steps = 0; steps <= tree.n_nodes; ++steps) {
        const int feature = tree.nodes[n].feature;
        if (feature < 0) { k = tree.nodes[n].klass; break; }
        n = ((double)s_f[feature] <= tree.nodes[n].threshold) ? tree.nodes[n].left : tree.nodes[n].right;
    }
    k = (k >= 0 && k < SEER_NUM_DIRECT_KERNELS) ? k : SEER_CSR_MP;
    if (sel) {
        sel->kernel_id = k;
        sel->valid = 1;
        sel->rows = rows; sel->cols = cols; sel->nnz = nnz;
        sel->max_len = s->mx; sel->min_len = s->mn;
        sel->sum_sq = s->sq; sel->empty = s->em;
#pragma unroll
        for (int i = 0; i < SEER_NUM_FEATURES; ++i) sel->f[i] = s_f[i];
    }
    return k;
}

// ---- selection from the flattened tree (depth <= 6), by the first wave of a workgroup.
// Walking the node array costs one dependent load from the kernel-argument memory per
// level (measured: 2.3 us of a 26 us step for a depth-6 tree).  Here every lane fetches one
// slot when the kernel starts, long before the statistics are ready; afterwards all
// comparisons are evaluated at once and the leaf is found with two ballots.
struct HeapRegs {
    int feature;
    double threshold;
    int klass_inner, klass_leaf;   // of slot lane, and of slot 63 + lane
};

__device__ __forceinline__ HeapRegs heap_load(const AutoHeap &h)
{
    const int l = threadIdx.x % kWave;
    return HeapRegs{h.feature[l], h.threshold[l], (int)h.klass[l], (int)h.klass[kHeapInternal + l]};
}

// All 64 lanes of one wave; s_f is the feature vector in LDS (complete and visible).
__device__ __forceinline__ int heap_walk(const HeapRegs &r, const float *s_f)
{
    const bool leaf = r.feature < 0;
    const bool right = !leaf && !((double)s_f[leaf ? 0 : r.feature] <= r.threshold);
    const uint64_t leaf_mask = __ballot(leaf), right_mask = __ballot(right);
    int i = 0;
#pragma unroll
    for (int d = 0; d < 6; ++d) {
        if ((leaf_mask >> i) & 1) break;              // i <= 62 here
        i = 2 * i + 1 + (int)((right_mask >> i) & 1);
    }
    const int k = i < kHeapInternal ? __shfl(r.klass_inner, i) : __shfl(r.klass_leaf, i - kHeapInternal);
    return (k >= 0 && k < SEER_NUM_DIRECT_KERNELS) ? k : SEER_CSR_MP;
}

__device__ __forceinline__ void write_selection(
    AutoSel *__restrict__ sel, int k, int rows, int cols, int64_t nnz, const FeatLds *s, const float *s_f)
{
    sel->kernel_id = k;
    sel->valid = 1;
    sel->rows = rows; sel->cols = cols; sel->nnz = nnz;
    sel->max_len = s->mx; sel->min_len = s->mn;
    sel->sum_sq = s->sq; sel->empty = s->em;
#pragma unroll
    for (int i = 0; i < SEER_NUM_FEATURES; ++i) sel->f[i] = s_f[i];
}

// The workgroup's statistics are in *s (after a barrier).  Derives the features (one lane),
// walks the flattened tree (first wave) and leaves the kernel id in *s_k for everyone; ends
// with a barrier.
__device__ __forceinline__ void select_with_heap(
    int rows, int cols, const int *__restrict__ rp, const FeatLds *s, float *s_f, const HeapRegs &hr,
    AutoSel *__restrict__ sel, int *s_k)
{
    int64_t nnz = 0;
    if (threadIdx.x == 0) {
        nnz = (int64_t)rp[rows] - (int64_t)rp[0];
        derive_features_device(rows, cols, nnz, s->mx, s->mn, (int64_t)s->em, s->sq, s_f);
    }
    __syncthreads();
    if (threadIdx.x < kWave) {
        const int k = heap_walk(hr, s_f);
        if (threadIdx.x == 0) {
            *s_k = k;
            if (sel) write_selection(sel, k, rows, cols, nnz, s, s_f);
        }
    }
    __syncthreads();
}

template <bool VEC>
__global__ __launch_bounds__(kFeatWG) void features_select_heap_kernel(
    int rows, int cols, const int *__restrict__ rp, const FeatPartial *__restrict__ part, uint32_t n_part,
    AutoSel *__restrict__ sel, const AutoHeap heap)
{
    __shared__ FeatLds s;
    __shared__ float s_f[SEER_NUM_FEATURES];
    __shared__ int s_k;
    HeapRegs hr{};
    if (threadIdx.x < kWave) hr = heap_load(heap);
    features_total<VEC>(rows, rp, part, n_part, &s);
    select_with_heap(rows, cols, rp, &s, s_f, hr, sel, &s_k);
}

template <bool VEC>
__global__ __launch_bounds__(kFeatWG) void features_select_kernel(
    int rows, int cols, const int *__restrict__ rp, const FeatPartial *__restrict__ part, uint32_t n_part,
    AutoSel *__restrict__ sel, const AutoTree tree)
{
    __shared__ FeatLds s;
    __shared__ float s_f[SEER_NUM_FEATURES];
    features_total<VEC>(rows, rp, part, n_part, &s);
    if (threadIdx.x == 0) select_on_device(rows, cols, rp, &s, s_f, tree, sel);
}

static_assert(kFeatMaxParts * sizeof(FeatPartial) <= kAutoSelOffset && sizeof(AutoSel) <= kAutoCarryOffset - kAutoSelOffset,
              "workspace layout");

constexpr int kAutoLdsMpBm = mp_lds_words<kMpIptLarge>() > bm_lds_words<kBmChunk>() ? mp_lds_words<kMpIptLarge>()
                                                                                     : bm_lds_words<kBmChunk>();
constexpr int kAutoLds = kAutoLdsMpBm > bm_lds_words<kWoChunkLarge>() + 2 ? kAutoLdsMpBm
                                                                           : bm_lds_words<kWoChunkLarge>() + 2;
static_assert(bm_lds_words<kWoChunk>() + 2 <= kAutoLds, "CSR,WO's products and its two bounds share the overlay");

// This workgroup's share of schedule k (the same k in every workgroup of the grid).
template <int IPT, bool VEC>
__device__ __forceinline__ void auto_dispatch(
    int k, int rows, int nnz, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    int *__restrict__ carry_row, float *__restrict__ carry_val, const AutoShape &shape, int remap, int *smem)
{
    static_assert(mp_lds_words<IPT>() <= kAutoLds, "LDS overlay too small");
    const uint32_t n_tiles = shape.tiles[k];
    if (k == SEER_CSR_WM) {
        // The one schedule whose tiles can outnumber the grid (launch_auto caps its share):
        // a workgroup takes every gridDim-th block position; tile_of_block is one-to-one
        // on [0, span), so each tile is still visited exactly once.
        const uint32_t span = remap ? tiles_per_xcd(n_tiles) * kXCD : n_tiles;
        for (uint32_t vb = blockIdx.x; vb < span; vb += gridDim.x) {
            const uint32_t t = tile_of_block(vb, n_tiles, remap);
            if (t >= n_tiles) continue;
            switch (shape.wm_lanes) {
            case 2: wm_body<2>(rows, rp, ci, va, x, y, t); break;
            case 4: wm_body<4>(rows, rp, ci, va, x, y, t); break;
            case 8: wm_body<8>(rows, rp, ci, va, x, y, t); break;
            case 16: wm_body<16>(rows, rp, ci, va, x, y, t); break;
            case 32: wm_body<32>(rows, rp, ci, va, x, y, t); break;
            default: wm_body<64>(rows, rp, ci, va, x, y, t); break;
            }
        }
        return;
    }
    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, k == SEER_CSR_TM ? (remap && shape.tm_remap) : remap);
    if (tile >= n_tiles) return;
    if (k == SEER_CSR_TM) {
        if (shape.tm_pair) tm_body<true, 2>(rows, nnz, rp, ci, va, x, y, tile);
        else if (shape.tm_short) tm_body<true>(rows, nnz, rp, ci, va, x, y, tile);
        else tm_body<false>(rows, nnz, rp, ci, va, x, y, tile);
    } else if (k == SEER_CSR_BM) {
        if (shape.bm_rows <= (int)kWoGroupRows)
            bm_body<kBmChunk, VEC, true, true, false, true, 256>(rows, rp, ci, va, x, y, shape.bm_rows,
                                                                 shape.bm_own_shift, tile, reinterpret_cast<float *>(smem));
        else   // (the host keeps bm_rows within kAutoBmMaxRows here)
            bm_body<kBmChunk, VEC, true, true, false, false, kAutoBmMaxRows>(rows, rp, ci, va, x, y, shape.bm_rows,
                                                                             shape.bm_own_shift, tile, reinterpret_cast<float *>(smem));
    } else if (k == SEER_CSR_WO) {
        if (wo_chunk_of(nnz) == kWoChunkLarge)
            wo_body<kWoChunkLarge, VEC, true>(rows, nnz, rp, ci, va, x, y, carry_row, carry_val, tile,
                                              reinterpret_cast<float *>(smem),
                                              reinterpret_cast<uint32_t *>(smem) + bm_lds_words<kWoChunkLarge>());
        else
            wo_body<kWoChunk, VEC, true>(rows, nnz, rp, ci, va, x, y, carry_row, carry_val, tile,
                                         reinterpret_cast<float *>(smem),
                                         reinterpret_cast<uint32_t *>(smem) + bm_lds_words<kWoChunk>());
    } else {
        mp_body<IPT, VEC, true>(rows, nnz, rp, ci, va, x, y, carry_row, carry_val, tile, smem);
    }
}

template <int IPT, bool VEC>
__global__ __launch_bounds__(kWG) void spmv_auto_kernel(
    int rows, int nnz, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    int *__restrict__ carry_row, float *__restrict__ carry_val, const AutoSel *__restrict__ sel,
    const AutoShape shape, int remap)
{
    __shared__ __attribute__((aligned(16))) int smem[kAutoLds];
    auto_dispatch<IPT, VEC>(sel->kernel_id, rows, nnz, rp, ci, va, x, y, carry_row, carry_val, shape, remap, smem);
}

// Selection inside the product's launch, for grids of a few hundred workgroups.  Every
// workgroup finishes the feature reduction for itself -- for a small matrix it reduces
// the whole row_ptr (n_part == 0; at most kAutoFusedRows offsets, out of L2 after the
// first workgroup touched them), for a larger one it folds the few partials a first
// pass left -- derives the same feature vector, walks the same tree and then runs its
// share of the chosen schedule.  The redundant work costs each workgroup two to three
// microseconds; a separate selection launch costs the whole path four to five.
// (With thousands of workgroups the redundant work adds up to more than the launch it
// saves -- measured on a 1M-row matrix: 37 us per step against 27.6 -- so larger grids
// keep the selection as a launch of its own.)
// Workgroup 0 leaves the record for seer_spmv_auto_result and the fix-up kernel.
template <int IPT, bool VEC, bool RPVEC>
__global__ __launch_bounds__(kWG) void spmv_auto_fused_kernel(
    int rows, int cols, int nnz, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    int *__restrict__ carry_row, float *__restrict__ carry_val, const FeatPartial *__restrict__ part,
    uint32_t n_part, AutoSel *__restrict__ sel, const AutoHeap heap, const AutoShape shape, int remap)
{
    __shared__ __attribute__((aligned(16))) int smem[kAutoLds];
    __shared__ FeatLds s;
    __shared__ float s_f[SEER_NUM_FEATURES];
    __shared__ int s_k;
    HeapRegs hr{};
    if (threadIdx.x < kWave) hr = heap_load(heap);
    int32_t mx, mn;
    uint64_t sq, em;
    if (n_part == 0) {
        features_accumulate_strided<RPVEC>(rows, rp, threadIdx.x, kWG, mx, mn, sq, em);
    } else {
        mx = INT32_MIN; mn = INT32_MAX; sq = 0; em = 0;
        for (uint32_t b = threadIdx.x; b < n_part; b += kWG) {
            const FeatPartial p = part[b];
            mx = max(mx, p.max_len);
            mn = min(mn, p.min_len);
            sq += p.sum_sq;
            em += p.empty;
        }
    }
    features_block_fold(mx, mn, sq, em, &s);
    select_with_heap(rows, cols, rp, &s, s_f, hr, blockIdx.x == 0 ? sel : nullptr, &s_k);
    auto_dispatch<IPT, VEC>(s_k, rows, nnz, rp, ci, va, x, y, carry_row, carry_val, shape, remap, smem);
}

__global__ __launch_bounds__(kWG) void spmv_auto_fixup_kernel(
    int rows, uint32_t n_mp, uint32_t n_wo, const int *__restrict__ carry_row,
    const float *__restrict__ carry_val, float *__restrict__ y, const AutoSel *__restrict__ sel)
{
    const int k = sel->kernel_id;
    if (k != SEER_CSR_MP && k != SEER_CSR_WO) return;
    mp_fixup_body(rows, k == SEER_CSR_MP ? n_mp : n_wo, carry_row, carry_val, y);
}

size_t auto_workspace_bytes(int rows, int nnz)
{
    const size_t mp = mp_workspace_bytes(rows, nnz, kMpIptSmall);
    const size_t wo = carry_workspace_bytes(wo_num_tiles(rows, nnz));
    return kAutoCarryOffset + (mp > wo ? mp : wo);
}

void launch_auto(const SpmvArgs &a, const AutoTree &tree, const AutoHeap *heap, const AutoShape &shape, bool vec,
                 int fused_rows, int fused_grid, void *workspace, hipStream_t st)
{
    char *ws = static_cast<char *>(workspace);
    FeatPartial *part = reinterpret_cast<FeatPartial *>(ws);
    AutoSel *sel = reinterpret_cast<AutoSel *>(ws + kAutoSelOffset);
    const uint32_t n_mp = shape.tiles[SEER_CSR_MP], n_wo = shape.tiles[SEER_CSR_WO];
    const uint32_t n_carry = n_mp > n_wo ? n_mp : n_wo;
    const size_t one = carry_workspace_bytes(n_carry) / 2;
    int *carry_row = reinterpret_cast<int *>(ws + kAutoCarryOffset);
    float *carry_val = reinterpret_cast<float *>(ws + kAutoCarryOffset + one);

    // One workgroup per tile of the schedule with the most tiles -- except CSR,WM, whose
    // tiles (64/G rows per wave) can be several times the others': beyond kAutoWmGrid
    // workgroups its share is capped at the others' maximum and its workgroups loop, so a
    // grid that runs another schedule does not launch thousands of workgroups to no purpose.
    uint32_t grid = 0, wm_grid = 0;
    for (int k = 0; k < SEER_NUM_DIRECT_KERNELS; ++k) {
        const uint32_t g = a.remap ? tiles_per_xcd(shape.tiles[k]) * kXCD : shape.tiles[k];
        if (k == SEER_CSR_WM) wm_grid = g;
        else grid = g > grid ? g : grid;
    }
    {
        const uint32_t cap = grid > kAutoWmGrid ? grid : kAutoWmGrid;
        const uint32_t g = wm_grid < cap ? wm_grid : cap;
        grid = g > grid ? g : grid;
    }
    const bool rp_vec = (reinterpret_cast<uintptr_t>(a.rp) & 15u) == 0;
    if (heap && grid <= (uint32_t)fused_grid) {
        // one launch for a small matrix; else a first pass that leaves a few partials
        uint32_t n_part = 0;
        if (a.rows > fused_rows) {
            n_part = features_num_parts(a.rows);
            n_part = n_part > kAutoFusedParts ? kAutoFusedParts : (n_part ? n_part : 1u);
            if (rp_vec)
                hipLaunchKernelGGL(features_partial_kernel<true>, dim3(n_part), dim3(kFeatPartWG), 0, st, a.rows, a.rp, part);
            else
                hipLaunchKernelGGL(features_partial_kernel<false>, dim3(n_part), dim3(kFeatPartWG), 0, st, a.rows, a.rp, part);
        }
#define SEER_FUSED_LAUNCH(I, V, R)                                                                          \
    hipLaunchKernelGGL((spmv_auto_fused_kernel<I, V, R>), dim3(grid), dim3(kWG), 0, st, a.rows, a.cols, a.nnz, \
                       a.rp, a.ci, a.va, a.x, a.y, carry_row, carry_val, part, n_part, sel, *heap, shape, a.remap)
        if (shape.mp_ipt == kMpIptSmall) {
            if (vec) { if (rp_vec) SEER_FUSED_LAUNCH(kMpIptSmall, true, true); else SEER_FUSED_LAUNCH(kMpIptSmall, true, false); }
            else     { if (rp_vec) SEER_FUSED_LAUNCH(kMpIptSmall, false, true); else SEER_FUSED_LAUNCH(kMpIptSmall, false, false); }
        } else {
            if (vec) { if (rp_vec) SEER_FUSED_LAUNCH(kMpIptLarge, true, true); else SEER_FUSED_LAUNCH(kMpIptLarge, true, false); }
            else     { if (rp_vec) SEER_FUSED_LAUNCH(kMpIptLarge, false, true); else SEER_FUSED_LAUNCH(kMpIptLarge, false, false); }
        }
#undef SEER_FUSED_LAUNCH
        hipLaunchKernelGGL(spmv_auto_fixup_kernel, dim3((n_carry + kWG - 1) / kWG), dim3(kWG), 0, st, a.rows, n_mp,
                           n_wo, carry_row, carry_val, a.y, sel);
        return;
    }

    const uint32_t n_part = features_num_parts(a.rows);
    if (rp_vec) {
        if (n_part)
            hipLaunchKernelGGL(features_partial_kernel<true>, dim3(n_part), dim3(kFeatPartWG), 0, st, a.rows, a.rp, part);
        if (heap)
            hipLaunchKernelGGL(features_select_heap_kernel<true>, dim3(1), dim3(kFeatWG), 0, st, a.rows, a.cols, a.rp,
                               part, n_part, sel, *heap);
        else
            hipLaunchKernelGGL(features_select_kernel<true>, dim3(1), dim3(kFeatWG), 0, st, a.rows, a.cols, a.rp, part,
                               n_part, sel, tree);
    } else {
        if (n_part)
            hipLaunchKernelGGL(features_partial_kernel<false>, dim3(n_part), dim3(kFeatPartWG), 0, st, a.rows, a.rp, part);
        if (heap)
            hipLaunchKernelGGL(features_select_heap_kernel<false>, dim3(1), dim3(kFeatWG), 0, st, a.rows, a.cols, a.rp,
                               part, n_part, sel, *heap);
        else
            hipLaunchKernelGGL(features_select_kernel<false>, dim3(1), dim3(kFeatWG), 0, st, a.rows, a.cols, a.rp, part,
                               n_part, sel, tree);
    }

#define SEER_AUTO_LAUNCH(I, V)                                                                             \
    hipLaunchKernelGGL((spmv_auto_kernel<I, V>), dim3(grid), dim3(kWG), 0, st, a.rows, a.nnz, a.rp, a.ci, \
                       a.va, a.x, a.y, carry_row, carry_val, sel, shape, a.remap)
    if (shape.mp_ipt == kMpIptSmall) {
        if (vec) SEER_AUTO_LAUNCH(kMpIptSmall, true); else SEER_AUTO_LAUNCH(kMpIptSmall, false);
    } else {
        if (vec) SEER_AUTO_LAUNCH(kMpIptLarge, true); else SEER_AUTO_LAUNCH(kMpIptLarge, false);
    }
#undef SEER_AUTO_LAUNCH
    hipLaunchKernelGGL(spmv_auto_fixup_kernel, dim3((n_carry + kWG - 1) / kWG), dim3(kWG), 0, st, a.rows, n_mp,
                       n_wo, carry_row, carry_val, a.y, sel);
}

} // namespace seer
