// The whole runtime flow of Sec. III-B -- gather features, evaluate the decision tree,
// run the chosen kernel -- as a few launches with no host round trip in between:
//
//   1. the feature reduction (one launch for a small matrix, two for a large one);
//      its finishing launch -- a single wave after a first pass, a workgroup for a small
//      matrix -- derives the feature vector on the device, walks the tree (handed over by
//      value in the kernel arguments) and leaves the chosen kernel id in device memory;
//   2. spmv_auto_kernel: one kernel that contains the five CSR schedules that need no
//      preprocessing; every workgroup reads the chosen id and runs that schedule's
//      body (the grid is sized for the reachable schedule that needs the most workgroups,
//      the rest exit);
//   3. spmv_auto_fixup_kernel: the carry fix-up of merge path and of the nonzero
//      split; exits at once unless one of them was chosen, and is not enqueued at all if
//      the host can tell from rows, cols and nnz that the tree cannot answer either.
// When the product's grid is small, steps 1 and 2 share a launch (or, for a small
// matrix, are one launch): see spmv_auto_fused_kernel.  When the known features leave the
// tree a single answer, step 1 is dropped: see spmv_auto_decided_kernel.
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
    uint32_t reachable, AutoSel *__restrict__ sel)
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
    if (!((reachable >> k) & 1u)) k = __ffs((int)reachable) - 1;   // (see select_in_wave)
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

// Entry `l` of the feature vector (l < SEER_NUM_FEATURES; other lanes get 1).  The same
// operations as derive_features_device, arranged so that every lane of a wave runs the same
// instructions on its own operands: f[l] = fl32((a / b) / c) with b, c = 1 where the entry
// has fewer divisions (x / 1 is exact), so the thirteen entries cost two fp64 divisions
// instead of seven one after the other.  rows > 0.
__device__ __forceinline__ float derive_feature_lane(int rows, int cols, int64_t nnz, const FeatTotals &t, int l)
{
    const double R = (double)(int64_t)rows, C = (double)(int64_t)cols, N = (double)nnz;
    const unsigned __int128 num = (unsigned __int128)(uint64_t)rows * (unsigned __int128)t.sq -
                                  (unsigned __int128)(uint64_t)nnz * (unsigned __int128)(uint64_t)nnz;
    const double VN = u128_to_double(num), RR = (double)((uint64_t)rows * (uint64_t)rows);
    const double MX = (double)(int64_t)t.mx, MN = (double)(int64_t)t.mn, E = (double)(int64_t)t.em;
    const bool density = l >= SEER_F_MEAN_DENSITY && l <= SEER_F_VAR_DENSITY;
    double a = 1.0, b = 1.0, c = 1.0;           // SEER_F_ITERATIONS: 1 on this path
    if (l == SEER_F_ROWS) a = R;
    if (l == SEER_F_COLS) a = C;
    if (l == SEER_F_NNZ || l == SEER_F_MEAN_LEN || l == SEER_F_MEAN_DENSITY) a = N;
    if (l == SEER_F_MAX_LEN || l == SEER_F_MAX_DENSITY) a = MX;
    if (l == SEER_F_MIN_LEN || l == SEER_F_MIN_DENSITY) a = MN;
    if (l == SEER_F_VAR_LEN || l == SEER_F_VAR_DENSITY) a = VN;
    if (l == SEER_F_EMPTY_FRAC) a = E;
    if (l == SEER_F_MEAN_LEN || l == SEER_F_EMPTY_FRAC || l == SEER_F_MEAN_DENSITY) b = R;
    if (l == SEER_F_VAR_LEN || l == SEER_F_VAR_DENSITY) b = RR;
    if (density) c = l == SEER_F_VAR_DENSITY ? C * C : C;
    if (density && cols <= 0) { a = 0.0; b = 1.0; c = 1.0; }   // no columns: densities are 0
    return (float)((a / b) / c);
}

// All 64 lanes of one wave, each holding its slot of the flattened tree in `r` and, for
// lane < SEER_NUM_FEATURES, its entry of the feature vector in `f`.
__device__ __forceinline__ int heap_walk_lanes(const HeapRegs &r, float f)
{
    const bool leaf = r.feature < 0;
    const float fv = __shfl(f, leaf ? 0 : r.feature);
    const bool right = !leaf && !((double)fv <= r.threshold);
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

// One wave: from the matrix's statistics to the kernel id (the same in every lane), and, if
// `sel` is given, the record seer_spmv_auto_result reads.  `reachable` has a bit per kernel
// id the host found reachable from rows, cols and nnz alone and sized the grid for; the
// device arrives at one of them unless nnz is not what row_ptr says, and then takes the
// lowest of them rather than a schedule the grid cannot hold.
__device__ __forceinline__ int select_in_wave(
    int rows, int cols, int64_t nnz, const FeatTotals &t, const HeapRegs &hr, uint32_t reachable,
    AutoSel *__restrict__ sel)
{
    const int l = threadIdx.x % kWave;
    const float f = derive_feature_lane(rows, cols, nnz, t, l);
    int k = heap_walk_lanes(hr, f);
    if (!((reachable >> k) & 1u)) k = __ffs((int)reachable) - 1;
    if (sel) {
        if (l < SEER_NUM_FEATURES) sel->f[l] = f;
        if (l == 0) {
            sel->kernel_id = k;
            sel->valid = 1;
            sel->rows = rows; sel->cols = cols; sel->nnz = nnz;
            sel->max_len = t.mx; sel->min_len = t.mn;
            sel->sum_sq = t.sq; sel->empty = t.em;
        }
    }
    return k;
}

// Finishing launch of the selection after a first pass: ONE wave folds the partials, derives
// the features, walks the tree and leaves the record -- no LDS, no barrier (as a workgroup of
// 1024 lanes that met in LDS atomics it took 4.4 us on the timeline).
__global__ __launch_bounds__(kWave) void features_select_wave_kernel(
    int rows, int cols, const int *__restrict__ rp, const FeatPartial *__restrict__ part, uint32_t n_part,
    AutoSel *__restrict__ sel, const AutoHeap heap, uint32_t reachable)
{
    const HeapRegs hr = heap_load(heap);
    const int64_t nnz = (int64_t)rp[rows] - (int64_t)rp[0];
    const FeatTotals t = fold_partials_wave(part, n_part);
    select_in_wave(rows, cols, nnz, t, hr, reachable, sel);
}

// Finishing launch of the selection when it is a launch of its own: the workgroup folds the
// partials of the first pass (or, for a small matrix, reduces row_ptr itself), its first wave
// derives the features, walks the tree and leaves the record.
template <bool VEC>
__global__ __launch_bounds__(kFeatWG) void features_select_heap_kernel(
    int rows, int cols, const int *__restrict__ rp, const FeatPartial *__restrict__ part, uint32_t n_part,
    AutoSel *__restrict__ sel, const AutoHeap heap, uint32_t reachable)
{
    __shared__ FeatLds s;
    HeapRegs hr{};
    int64_t nnz = 0;
    if (threadIdx.x < kWave) {                       // requested before the reduction, used after it
        hr = heap_load(heap);
        nnz = (int64_t)rp[rows] - (int64_t)rp[0];
    }
    features_total<VEC>(rows, rp, part, n_part, &s);
    if (threadIdx.x < kWave) select_in_wave(rows, cols, nnz, FeatTotals{s.mx, s.mn, s.sq, s.em}, hr, reachable, sel);
}

template <bool VEC>
__global__ __launch_bounds__(kFeatWG) void features_select_kernel(
    int rows, int cols, const int *__restrict__ rp, const FeatPartial *__restrict__ part, uint32_t n_part,
    AutoSel *__restrict__ sel, const AutoTree tree, uint32_t reachable)
{
    __shared__ FeatLds s;
    __shared__ float s_f[SEER_NUM_FEATURES];
    features_total<VEC>(rows, rp, part, n_part, &s);
    if (threadIdx.x == 0) select_on_device(rows, cols, rp, &s, s_f, tree, reachable, sel);
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

// The product when the host could decide alone: every leaf the tree can reach from rows,
// cols and nnz names the same kernel, so nothing is gathered.  Workgroup 0 leaves the record
// (valid = 2: no statistics, known features only).
template <int IPT, bool VEC>
__global__ __launch_bounds__(kWG) void spmv_auto_decided_kernel(
    int rows, int nnz, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    int *__restrict__ carry_row, float *__restrict__ carry_val, AutoSel *__restrict__ sel,
    const AutoSel record, const AutoShape shape, int remap)
{
    __shared__ __attribute__((aligned(16))) int smem[kAutoLds];
    if (blockIdx.x == 0 && threadIdx.x == 0) *sel = record;
    auto_dispatch<IPT, VEC>(record.kernel_id, rows, nnz, rp, ci, va, x, y, carry_row, carry_val, shape, remap, smem);
}

// Selection inside the product's launch.  The first wave of every workgroup finishes the
// feature reduction for itself -- it folds the up to 64 partials a first pass left (lane <->
// partial, no LDS; for a matrix of at most kAutoFusedRows rows there is no first pass and the
// whole workgroup reduces row_ptr, out of L2 after the first workgroup touched it) -- derives
// the same feature vector, walks the same tree, and hands the kernel id to the other waves
// through LDS; then the workgroup runs its share of the chosen schedule.  The redundant work
// is a few hundred instructions of one wave behind one load of two kilobytes that hits L2,
// while a selection launch costs the path about three microseconds.  Workgroup 0 leaves the
// record for seer_spmv_auto_result and the fix-up kernel.
// Used for grids of up to about a thousand workgroups.  Beyond, it was measured slower than
// the separate launch (a 54 MB stencil: 24.4 us per step against 22.8; the product itself
// 17.2 against 13.0 us, and a first pass of 64 fat workgroups 6.3 against 4.6 us for 512).
template <int IPT, bool VEC, bool RPVEC>
__global__ __launch_bounds__(kWG) void spmv_auto_fused_kernel(
    int rows, int cols, int nnz, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    int *__restrict__ carry_row, float *__restrict__ carry_val, const FeatPartial *__restrict__ part,
    uint32_t n_part, AutoSel *__restrict__ sel, const AutoHeap heap, const AutoShape shape, int remap)
{
    __shared__ __attribute__((aligned(16))) int smem[kAutoLds];
    __shared__ FeatLds s;
    __shared__ int s_k;
    const bool first_wave = threadIdx.x < kWave;
    HeapRegs hr{};
    int64_t nnz_dev = 0;
    FeatTotals t{INT32_MIN, INT32_MAX, 0, 0};
    if (first_wave) {
        hr = heap_load(heap);
        nnz_dev = (int64_t)rp[rows] - (int64_t)rp[0];
    }
    if (n_part == 0) {                                // block-uniform
        features_accumulate_strided<RPVEC>(rows, rp, threadIdx.x, kWG, t.mx, t.mn, t.sq, t.em);
        features_block_fold(t.mx, t.mn, t.sq, t.em, &s);
        t = FeatTotals{s.mx, s.mn, s.sq, s.em};
    } else if (first_wave) {
        t = fold_partials_wave(part, n_part);
    }
    if (first_wave) {
        const int k = select_in_wave(rows, cols, nnz_dev, t, hr, shape.reachable, blockIdx.x == 0 ? sel : nullptr);
        if (threadIdx.x == 0) s_k = k;
    }
    __syncthreads();
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

// The first pass ahead of a product that selects for itself: at most kAutoFusedParts
// partials, sixteen rows (four 16-byte loads in flight) per lane and trip; workgroups of
// 1024 lanes once 256-lane ones would need more than one trip.
static uint32_t launch_fused_partials(const SpmvArgs &a, FeatPartial *part, bool rp_vec, hipStream_t st)
{
    const uint32_t rows = (uint32_t)a.rows;
    if (rows <= kAutoFusedParts * kFeatPartWG * 16u) {
        const uint32_t n = (rows + kFeatPartWG * 16u - 1u) / (kFeatPartWG * 16u);
        if (rp_vec) hipLaunchKernelGGL((features_partial_kernel<true, kFeatPartWG>), dim3(n), dim3(kFeatPartWG), 0, st, a.rows, a.rp, part);
        else hipLaunchKernelGGL((features_partial_kernel<false, kFeatPartWG>), dim3(n), dim3(kFeatPartWG), 0, st, a.rows, a.rp, part);
        return n;
    }
    uint32_t n = (rows + kFeatWG * 16u - 1u) / (kFeatWG * 16u);
    n = n > kAutoFusedParts ? kAutoFusedParts : n;
    if (rp_vec) hipLaunchKernelGGL((features_partial_kernel<true, kFeatWG>), dim3(n), dim3(kFeatWG), 0, st, a.rows, a.rp, part);
    else hipLaunchKernelGGL((features_partial_kernel<false, kFeatWG>), dim3(n), dim3(kFeatWG), 0, st, a.rows, a.rp, part);
    return n;
}

void launch_auto(const SpmvArgs &a, const AutoTree &tree, const AutoHeap *heap, const AutoShape &shape, bool vec,
                 const AutoPolicy &policy, const AutoSel *decided, void *workspace, hipStream_t st)
{
    char *ws = static_cast<char *>(workspace);
    FeatPartial *part = reinterpret_cast<FeatPartial *>(ws);
    AutoSel *sel = reinterpret_cast<AutoSel *>(ws + kAutoSelOffset);
    const uint32_t n_mp = shape.tiles[SEER_CSR_MP], n_wo = shape.tiles[SEER_CSR_WO];
    const uint32_t n_carry = n_mp > n_wo ? n_mp : n_wo;
    const size_t one = carry_workspace_bytes(n_carry) / 2;
    int *carry_row = reinterpret_cast<int *>(ws + kAutoCarryOffset);
    float *carry_val = reinterpret_cast<float *>(ws + kAutoCarryOffset + one);
    const auto reachable = [&](int k) { return ((shape.reachable >> k) & 1u) != 0; };

    // One workgroup per tile of the reachable schedule with the most tiles -- except CSR,WM,
    // whose tiles (64/G rows per wave) can be several times the others': beyond kAutoWmGrid
    // workgroups its share is capped at the others' maximum and its workgroups loop, so a
    // grid that runs another schedule does not launch thousands of workgroups to no purpose.
    uint32_t grid = 0, wm_grid = 0;
    for (int k = 0; k < SEER_NUM_DIRECT_KERNELS; ++k) {
        if (!reachable(k)) continue;
        const uint32_t g = a.remap ? tiles_per_xcd(shape.tiles[k]) * kXCD : shape.tiles[k];
        if (k == SEER_CSR_WM) wm_grid = g;
        else grid = g > grid ? g : grid;
    }
    if (reachable(SEER_CSR_WM)) {
        const uint32_t cap = grid > kAutoWmGrid ? grid : kAutoWmGrid;
        const uint32_t g = wm_grid < cap ? wm_grid : cap;
        grid = g > grid ? g : grid;
    }
    // The fix-up launch finds nothing to do unless merge path or the nonzero split ran: it
    // is only enqueued if the tree can get to one of them from what the host knows.
    const bool carries = reachable(SEER_CSR_MP) || reachable(SEER_CSR_WO);

    if (decided) {
#define SEER_DECIDED_LAUNCH(I, V)                                                                          \
    hipLaunchKernelGGL((spmv_auto_decided_kernel<I, V>), dim3(grid), dim3(kWG), 0, st, a.rows, a.nnz, a.rp, \
                       a.ci, a.va, a.x, a.y, carry_row, carry_val, sel, *decided, shape, a.remap)
        if (shape.mp_ipt == kMpIptSmall) {
            if (vec) SEER_DECIDED_LAUNCH(kMpIptSmall, true); else SEER_DECIDED_LAUNCH(kMpIptSmall, false);
        } else {
            if (vec) SEER_DECIDED_LAUNCH(kMpIptLarge, true); else SEER_DECIDED_LAUNCH(kMpIptLarge, false);
        }
#undef SEER_DECIDED_LAUNCH
        if (carries)
            launch_carry_fixup(a.rows, decided->kernel_id == SEER_CSR_MP ? n_mp : n_wo, carry_row, carry_val, a.y, st);
        return;
    }

    const bool rp_vec = (reinterpret_cast<uintptr_t>(a.rp) & 15u) == 0;
    if (heap && (grid <= (uint32_t)policy.fused_grid || a.rows <= policy.fused_max_rows)) {
        // one launch for a small matrix; else a first pass that leaves a few partials
        const uint32_t n_part = a.rows > policy.fused_rows ? launch_fused_partials(a, part, rp_vec, st) : 0u;
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
        if (carries)
            hipLaunchKernelGGL(spmv_auto_fixup_kernel, dim3((n_carry + kWG - 1) / kWG), dim3(kWG), 0, st, a.rows, n_mp,
                               n_wo, carry_row, carry_val, a.y, sel);
        return;
    }

    const uint32_t n_part = features_num_parts(a.rows, policy.part_rows);
    if (rp_vec) {
        if (n_part)
            hipLaunchKernelGGL(features_partial_kernel<true>, dim3(n_part), dim3(kFeatPartWG), 0, st, a.rows, a.rp, part);
        if (heap && n_part && policy.select_wave)
            hipLaunchKernelGGL(features_select_wave_kernel, dim3(1), dim3(kWave), 0, st, a.rows, a.cols, a.rp, part,
                               n_part, sel, *heap, shape.reachable);
        else if (heap)
            hipLaunchKernelGGL(features_select_heap_kernel<true>, dim3(1), dim3(kFeatWG), 0, st, a.rows, a.cols, a.rp,
                               part, n_part, sel, *heap, shape.reachable);
        else
            hipLaunchKernelGGL(features_select_kernel<true>, dim3(1), dim3(kFeatWG), 0, st, a.rows, a.cols, a.rp, part,
                               n_part, sel, tree, shape.reachable);
    } else {
        if (n_part)
            hipLaunchKernelGGL(features_partial_kernel<false>, dim3(n_part), dim3(kFeatPartWG), 0, st, a.rows, a.rp, part);
        if (heap && n_part && policy.select_wave)
            hipLaunchKernelGGL(features_select_wave_kernel, dim3(1), dim3(kWave), 0, st, a.rows, a.cols, a.rp, part,
                               n_part, sel, *heap, shape.reachable);
        else if (heap)
            hipLaunchKernelGGL(features_select_heap_kernel<false>, dim3(1), dim3(kFeatWG), 0, st, a.rows, a.cols, a.rp,
                               part, n_part, sel, *heap, shape.reachable);
        else
            hipLaunchKernelGGL(features_select_kernel<false>, dim3(1), dim3(kFeatWG), 0, st, a.rows, a.cols, a.rp, part,
                               n_part, sel, tree, shape.reachable);
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
    if (carries)
        hipLaunchKernelGGL(spmv_auto_fixup_kernel, dim3((n_carry + kWG - 1) / kWG), dim3(kWG), 0, st, a.rows, n_mp,
                           n_wo, carry_row, carry_val, a.y, sel);
}

} // namespace seer
