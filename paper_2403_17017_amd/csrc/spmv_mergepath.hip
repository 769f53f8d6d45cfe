// CSR,MP -- the work-oriented schedule of Table II: the total work, nonzeros plus
// outputs (rows), is cut into equal shares regardless of how it falls into rows.
//
// The merge of the row-end offsets row_ptr[1..rows] with the nonzero indices
// 0..nnz-1 (a row end comes first on a tie) has rows + nnz items.  Row end i sits
// at merge position row_ptr[i+1] + i, so the number of row ends among the first D
// items is  #{ i : row_ptr[i+1] + i + 1 <= D },  a monotone predicate over i.
//
//  * A workgroup owns T = 256 * IPT consecutive items.  Waves 0 and 1 find the
//    tile's two corner coordinates with a 64-ary search over row_ptr (each lane
//    probes one position, a ballot counts the hits: 4 rounds for 16 M rows).
//  * The tile's row ends and its products val * x[col] (full-width coalesced loads)
//    are staged in one LDS array of T words.
//  * Each lane then owns IPT consecutive items: it binary-searches its start in
//    LDS and walks, adding products and emitting a row sum at every row end.
//  * The partial sum a lane is left with belongs to a row finished by a later lane:
//    a segmented scan over (emitted-a-row, partial) pairs delivers it.
//  * Row sums go back through LDS so that y is written with coalesced stores.
//  * What a tile is left with belongs to a row finished by a later tile: it is
//    stored as (row, partial) and a second small kernel adds, per row, the partials
//    of the tiles before the one that wrote y.  Summation order is fixed, so the
//    result is deterministic; y is not pre-zeroed and every row is written once.
#include "common.hiph"
#include "launch.h"

namespace seer {

// Row ends among the first D merge items; all 64 lanes of one wave cooperate and
// all return the same value.
__device__ __forceinline__ uint32_t diagonal_rows(uint32_t D, uint32_t rows, uint32_t nnz,
                                                  const int *__restrict__ rp, uint32_t lane)
{
    uint32_t lo = D > nnz ? D - nnz : 0u;   // rows below lo are certainly consumed
    uint32_t hi = D < rows ? D : rows;      // rows at or above hi certainly are not
    while (lo < hi) {
        const uint32_t step = (hi - lo + 63u) / 64u;
        const uint32_t p = lo + (lane + 1u) * step - 1u;
        const bool hit = p < hi && (uint32_t)rp[p + 1] + p + 1u <= D;
        const uint32_t c = (uint32_t)__popcll(__ballot(hit));   // hits form a prefix of the lanes
        const uint32_t nlo = lo + c * step;
        const uint32_t cap = lo + (c + 1u) * step - 1u;         // first probe that missed
        hi = cap < hi ? cap : hi;
        lo = nlo;
    }
    return lo;
}

struct SegPair {  // (some lane in the span emitted a row, sum since the last emit)
    int f;
    float v;
};
__device__ __forceinline__ SegPair seg_join(SegPair left, SegPair right)
{
    SegPair r;
    r.f = left.f | right.f;
    r.v = right.f ? right.v : left.v + right.v;
    return r;
}

template <int IPT, bool VEC, bool NT>
__global__ __launch_bounds__(kWG) void spmv_mp_kernel(
    int rows, int nnz, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    int *__restrict__ carry_row, float *__restrict__ carry_val, uint32_t n_tiles, int remap)
{
    static_assert(IPT % 2 == 1, "odd items per lane keeps the walk free of LDS bank conflicts");
    constexpr uint32_t T = kWG * IPT;
    constexpr int NV = (T + 3 + 4 * kWG - 1) / (4 * kWG);
    __shared__ int s_item[T];     // [0, nr): row ends relative to j0, later row sums; [nr, nr+nn): products
    __shared__ uint32_t s_coord[2];
    __shared__ int s_wf[kWG / kWave];
    __shared__ float s_wv[kWG / kWave];

    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;
    const uint32_t tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const uint32_t total = (uint32_t)rows + (uint32_t)nnz;
    const uint32_t d0 = tile * T;
    const uint32_t d1 = total - d0 > T ? d0 + T : total;

    if (wave < 2) {
        const uint32_t i = diagonal_rows(wave ? d1 : d0, (uint32_t)rows, (uint32_t)nnz, rp, lane);
        if (lane == 0) s_coord[wave] = i;
    }
    __syncthreads();
    const uint32_t i0 = s_coord[0], i1 = s_coord[1];
    const uint32_t j0 = d0 - i0, j1 = d1 - i1;
    const uint32_t nr = i1 - i0, nn = j1 - j0, n_items = d1 - d0;

    // ---- stage row ends and products
    for (uint32_t a = tid; a < nr; a += kWG) s_item[a] = (int)((uint32_t)load_1<NT>(rp + i0 + 1 + a) - j0);
    {
        const uint32_t base = j0 & ~3u;
        v4i c[NV];
        v4f v[NV];
        bool full[NV];
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            const uint32_t k = base + 4u * (tid + kWG * m);
            full[m] = VEC && k >= j0 && k + 4 <= j1;
            if (full[m]) {
                c[m] = load_v4i<NT>(ci + k);
                v[m] = load_v4f<NT>(va + k);
            }
        }
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            const uint32_t k = base + 4u * (tid + kWG * m);
            if (full[m]) {
                float *dst = reinterpret_cast<float *>(s_item + nr + (k - j0));
                dst[0] = v[m].x * x[c[m].x];
                dst[1] = v[m].y * x[c[m].y];
                dst[2] = v[m].z * x[c[m].z];
                dst[3] = v[m].w * x[c[m].w];
            } else {
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    const uint32_t j = k + q;
                    if (j >= j0 && j < j1)
                        reinterpret_cast<float *>(s_item)[nr + (j - j0)] = load_1<NT>(va + j) * x[load_1<NT>(ci + j)];
                }
            }
        }
    }
    __syncthreads();

    // ---- this lane's start inside the tile
    const uint32_t d = min(tid * IPT, n_items);
    const uint32_t dend = min(d + IPT, n_items);
    uint32_t a, b;
    {
        uint32_t lo = d > nn ? d - nn : 0u, hi = d < nr ? d : nr;
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if ((uint32_t)s_item[mid] + mid + 1u <= d) lo = mid + 1u; else hi = mid;
        }
        a = lo;
        b = d - lo;
    }
    const uint32_t a_first = a;

    // ---- walk: IPT items, sums kept in registers until every lane is done reading row ends
    float out[IPT];
    uint32_t emit_mask = 0;
    float acc = 0.f;
    uint32_t next_end = a < nr ? (uint32_t)s_item[a] : 0xFFFFFFFFu;
#pragma unroll
    for (int it = 0; it < IPT; ++it) {
        out[it] = 0.f;
        if (d + it < dend) {
            if (next_end <= b) {          // every product of row i0 + a has been taken
                out[it] = acc;
                emit_mask |= 1u << it;
                acc = 0.f;
                ++a;
                next_end = a < nr ? (uint32_t)s_item[a] : 0xFFFFFFFFu;
            } else {
                acc += reinterpret_cast<const float *>(s_item)[nr + b];
                ++b;
            }
        }
    }

    // ---- segmented scan of (emitted, leftover) across the workgroup
    SegPair incl{emit_mask != 0, acc};
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        SegPair left;
        left.f = __shfl_up(incl.f, off);
        left.v = __shfl_up(incl.v, off);
        if (lane >= (uint32_t)off) incl = seg_join(left, incl);
    }
    SegPair excl;   // join of all earlier lanes of this wave
    excl.f = __shfl_up(incl.f, 1);
    excl.v = __shfl_up(incl.v, 1);
    if (lane == 0) excl = SegPair{0, 0.f};
    if (lane == kWave - 1) {
        s_wf[wave] = incl.f;
        s_wv[wave] = incl.v;
    }
    __syncthreads();    // also: every lane has finished reading row ends
    SegPair before{0, 0.f};
    for (uint32_t w = 0; w < wave; ++w) before = seg_join(before, SegPair{s_wf[w], s_wv[w]});
    const float carry_in = seg_join(before, excl).v;

    // ---- row sums into the row-end slots, then coalesced store
    {
        uint32_t slot = a_first;
        bool first = true;
#pragma unroll
        for (int it = 0; it < IPT; ++it) {
            if (emit_mask & (1u << it)) {
                const float s = first ? out[it] + carry_in : out[it];
                first = false;
                reinterpret_cast<float *>(s_item)[slot++] = s;
            }
        }
    }
    if (tid == kWG - 1) {
        SegPair all = seg_join(before, incl);
        carry_row[tile] = (int)i1;          // == rows when the tile ends the matrix
        carry_val[tile] = all.v;
    }
    __syncthreads();
    for (uint32_t r = tid; r < nr; r += kWG) y[i0 + r] = reinterpret_cast<const float *>(s_item)[r];
}

// Adds to each row that spans tiles the partial sums of the tiles before the one
// that finished it.  carry_row is non-decreasing, so a row's partials are one run;
// the lane at the head of a run adds it up in tile order.
__global__ __launch_bounds__(kWG) void spmv_mp_fixup_kernel(
    int rows, uint32_t n_tiles, const int *__restrict__ carry_row,
    const float *__restrict__ carry_val, float *__restrict__ y)
{
    const uint32_t k = blockIdx.x * kWG + threadIdx.x;
    if (k >= n_tiles) return;
    const int r = carry_row[k];
    if (r >= rows) return;
    if (k > 0 && carry_row[k - 1] == r) return;
    float s = carry_val[k];
    for (uint32_t q = k + 1; q < n_tiles && carry_row[q] == r; ++q) s += carry_val[q];
    y[r] += s;
}

uint32_t mp_num_tiles(int rows, int nnz, int ipt)
{
    const uint64_t total = (uint64_t)rows + (uint64_t)nnz;
    const uint64_t T = (uint64_t)kWG * ipt;
    return (uint32_t)((total + T - 1) / T);
}

size_t mp_workspace_bytes(int rows, int nnz, int ipt)
{
    // carry_row then carry_val, each padded to a multiple of 256 bytes
    const size_t n = mp_num_tiles(rows, nnz, ipt);
    const size_t one = (n * 4 + 255) & ~(size_t)255;
    return 2 * one;
}

template <int IPT>
static void launch_mp_ipt(const SpmvArgs &a, bool vec, void *workspace, hipStream_t st)
{
    const uint32_t n_tiles = mp_num_tiles(a.rows, a.nnz, IPT);
    if (n_tiles == 0) return;
    const size_t one = ((size_t)n_tiles * 4 + 255) & ~(size_t)255;
    int *carry_row = static_cast<int *>(workspace);
    float *carry_val = reinterpret_cast<float *>(static_cast<char *>(workspace) + one);
    const dim3 grid(a.remap ? tiles_per_xcd(n_tiles) * kXCD : n_tiles);
#define SEER_MP_LAUNCH(V, N)                                                                            \
    hipLaunchKernelGGL((spmv_mp_kernel<IPT, V, N>), grid, dim3(kWG), 0, st, a.rows, a.nnz, a.rp, a.ci, a.va, \
                       a.x, a.y, carry_row, carry_val, n_tiles, a.remap)
    if (vec) {
        if (a.nt) SEER_MP_LAUNCH(true, true); else SEER_MP_LAUNCH(true, false);
    } else {
        if (a.nt) SEER_MP_LAUNCH(false, true); else SEER_MP_LAUNCH(false, false);
    }
#undef SEER_MP_LAUNCH
    hipLaunchKernelGGL(spmv_mp_fixup_kernel, dim3((n_tiles + kWG - 1) / kWG), dim3(kWG), 0, st,
                       a.rows, n_tiles, carry_row, carry_val, a.y);
}

void launch_mp(const SpmvArgs &a, int ipt, bool vec, void *workspace, hipStream_t st)
{
    if (ipt == kMpIptSmall) launch_mp_ipt<kMpIptSmall>(a, vec, workspace, st);
    else launch_mp_ipt<kMpIptLarge>(a, vec, workspace, st);
}

} // namespace seer
