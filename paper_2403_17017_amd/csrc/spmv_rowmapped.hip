// Row-mapped CSR SpMV schedules for gfx950 (Table II of the Seer case study):
//   CSR,TM  thread mapped     -- one row per lane
//   CSR,WM  wavefront mapped  -- one row per group of G lanes, 64/G rows per wave
//   CSR,BM  block mapped      -- a block of consecutive rows per workgroup; the
//                                block's contiguous nonzero range is streamed with
//                                full-width coalesced loads, products are staged in
//                                LDS and reduced per row from there
// All compute y_i = sum_k values[k] * x[col_idx[k]] over k in [row_ptr[i], row_ptr[i+1]).
#include "common.hiph"
#include "launch.h"

namespace seer {

// ------------------------------------------------------------------ CSR,TM
__global__ __launch_bounds__(kWG) void spmv_tm_kernel(
    int rows, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    uint32_t n_tiles, int remap)
{
    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;
    const uint32_t row = tile * kWG + threadIdx.x;
    if (row >= (uint32_t)rows) return;
    uint32_t k = (uint32_t)rp[row];
    const uint32_t e = (uint32_t)rp[row + 1];
    // four independent partial sums: keeps four gathers in flight and bounds the
    // rounding error of a long row to a quarter of a single running sum's
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    for (; k + 4 <= e; k += 4) {
        const int c0 = ci[k], c1 = ci[k + 1], c2 = ci[k + 2], c3 = ci[k + 3];
        const float v0 = va[k], v1 = va[k + 1], v2 = va[k + 2], v3 = va[k + 3];
        a0 += v0 * x[c0];
        a1 += v1 * x[c1];
        a2 += v2 * x[c2];
        a3 += v3 * x[c3];
    }
    for (; k < e; ++k) a0 += va[k] * x[ci[k]];
    y[row] = (a0 + a1) + (a2 + a3);
}

// ------------------------------------------------------------------ CSR,WM
template <int G>
__global__ __launch_bounds__(kWG) void spmv_wm_kernel(
    int rows, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    uint32_t n_tiles, int remap)
{
    constexpr uint32_t kRowsPerWG = kWG / G;
    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;                 // whole workgroup leaves together
    const uint32_t lg = threadIdx.x % G;         // lane inside the group
    const uint32_t row = tile * kRowsPerWG + threadIdx.x / G;
    const bool live = row < (uint32_t)rows;
    uint32_t k = 0, e = 0;
    if (live) {
        k = (uint32_t)rp[row] + lg;
        e = (uint32_t)rp[row + 1];
    }
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    for (; k + 3 * G < e; k += 4 * G) {
        const int c0 = ci[k], c1 = ci[k + G], c2 = ci[k + 2 * G], c3 = ci[k + 3 * G];
        const float v0 = va[k], v1 = va[k + G], v2 = va[k + 2 * G], v3 = va[k + 3 * G];
        a0 += v0 * x[c0];
        a1 += v1 * x[c1];
        a2 += v2 * x[c2];
        a3 += v3 * x[c3];
    }
    for (; k < e; k += G) a0 += va[k] * x[ci[k]];
    // every lane of the wave reaches this point (no early exit above for dead rows)
    const float s = group_sum<G>((a0 + a1) + (a2 + a3));
    if (live && lg == 0) y[row] = s;
}

// ------------------------------------------------------------------ CSR,BM
// A workgroup owns rows_per_block consecutive rows, i.e. one contiguous range of
// nonzeros [s, e).  The range is streamed in chunks of CH entries with 16-byte loads
// (entry k of the chunk is loaded by lane (k / 4) mod 256, whatever row it belongs
// to), the products val * x[col] are parked in LDS, and after one barrier each lane
// adds up the slice of the chunk that belongs to each of its rows.  A row whose
// slice is longer than kBmLong is instead reduced by the whole wave that owns it.
// Row bounds live in registers, so the only LDS traffic is the products.
//
// Ownership: with 256 or more rows per block, lane t owns rows t, t + 256, ...;
// with fewer, the rows are spread evenly over the 256 lanes (every 256/P-th lane
// owns one, P = rows per block rounded up to a power of two) so that all four waves
// share the per-row work.
// LDS index i is stored at i + i/32: a lane walking its row with a stride that is a
// multiple of 32 words would otherwise hit one bank with the whole wave.
constexpr int kBmLong = 128;

__device__ __forceinline__ uint32_t lds_pad(uint32_t i) { return i + (i >> 5); }

// Stage val * x[col] for entries [lo, ce) of the chunk starting at cs (cs % 4 == 0)
// into s_prod[lds_pad(k - cs)].  All loads are issued before the first gather.
template <int CH, bool VEC, bool NT>
__device__ __forceinline__ void stage_products(
    const int *__restrict__ ci, const float *__restrict__ va, const float *__restrict__ x,
    float *__restrict__ s_prod, uint32_t cs, uint32_t lo, uint32_t ce, int tid)
{
    constexpr int NV = CH / (4 * kWG);
    v4i c[NV];
    v4f v[NV];
    bool full[NV];
#pragma unroll
    for (int m = 0; m < NV; ++m) {
        const uint32_t k = cs + 4u * (uint32_t)(tid + kWG * m);
        full[m] = VEC && k >= lo && k + 4 <= ce;
        if (full[m]) {
            c[m] = load_v4i<NT>(ci + k);
            v[m] = load_v4f<NT>(va + k);
        }
    }
#pragma unroll
    for (int m = 0; m < NV; ++m) {
        const uint32_t k = cs + 4u * (uint32_t)(tid + kWG * m);
        if (full[m]) {
            float *dst = s_prod + lds_pad(k - cs);   // k - cs is a multiple of 4: no pad inside the quad
            dst[0] = v[m].x * x[c[m].x];
            dst[1] = v[m].y * x[c[m].y];
            dst[2] = v[m].z * x[c[m].z];
            dst[3] = v[m].w * x[c[m].w];
        } else {
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q) {
                const uint32_t j = k + q;
                if (j >= lo && j < ce) s_prod[lds_pad(j - cs)] = load_1<NT>(va + j) * x[load_1<NT>(ci + j)];
            }
        }
    }
}

template <int CH, bool VEC, bool NT>
__global__ __launch_bounds__(kWG) void spmv_bm_kernel(
    int rows, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    int rows_per_block, int own_shift, uint32_t n_tiles, int remap)
{
    static_assert(CH % (4 * kWG) == 0, "chunk must be whole 16-byte rounds");
    constexpr int RPT = kBmMaxRows / kWG;   // most rows one lane owns
    __shared__ float s_prod[CH + CH / 32];

    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;
    const int tid = (int)threadIdx.x, lane = tid % kWave;
    const uint32_t r0 = tile * (uint32_t)rows_per_block;
    const int nr = (int)min((uint32_t)rows_per_block, (uint32_t)rows - r0);

    const uint32_t s = (uint32_t)rp[r0], e = (uint32_t)rp[r0 + nr];   // block-uniform
    // lane's m-th row: ((tid >> own_shift) + 256 * m) if tid is a multiple of 2^own_shift
    // (own_shift > 0 only when rows_per_block < 256, and then m = 0 is the only one)
    const bool owner_lane = (tid & ((1 << own_shift) - 1)) == 0;
    const int row_base = tid >> own_shift;
    uint32_t ra[RPT], rb[RPT];
    float acc[RPT];
#pragma unroll
    for (int m = 0; m < RPT; ++m) {
        const int r = row_base + kWG * m;
        const bool own = owner_lane && r < nr;
        ra[m] = own ? (uint32_t)load_1<NT>(rp + r0 + r) : 0u;
        rb[m] = own ? (uint32_t)load_1<NT>(rp + r0 + r + 1) : 0u;
        acc[m] = 0.f;
    }

    for (uint32_t cs = s & ~3u; cs < e; cs += CH) {
        const uint32_t ce = min(cs + (uint32_t)CH, e);
        const uint32_t lo = max(cs, s);
        stage_products<CH, VEC, NT>(ci, va, x, s_prod, cs, lo, ce, tid);
        __syncthreads();
#pragma unroll
        for (int m = 0; m < RPT; ++m) {
            if (kWG * m >= nr) break;                       // block-uniform
            const uint32_t a = max(ra[m], lo), b = min(rb[m], ce);
            const bool has = b > a;
            const bool is_long = has && b - a > (uint32_t)kBmLong;
            if (has && !is_long) {
                float t = 0.f;
                for (uint32_t k = a; k < b; ++k) t += s_prod[lds_pad(k - cs)];
                acc[m] += t;
            }
            // rows that are long inside this chunk: the owning wave reduces them together
            uint64_t todo = __ballot(is_long);
            while (todo) {                                   // wave-uniform
                const int src = __ffsll((unsigned long long)todo) - 1;
                todo &= todo - 1;
                const uint32_t la = (uint32_t)__shfl((int)a, src), lb = (uint32_t)__shfl((int)b, src);
                float t = 0.f;
                for (uint32_t k = la + (uint32_t)lane; k < lb; k += kWave) t += s_prod[lds_pad(k - cs)];
                t = group_sum<64>(t);
                if (lane == src) acc[m] += t;
            }
        }
        if (ce < e) __syncthreads();   // s_prod is overwritten by the next chunk
    }
#pragma unroll
    for (int m = 0; m < RPT; ++m) {
        const int r = row_base + kWG * m;
        if (owner_lane && r < nr) y[r0 + r] = acc[m];
    }
}

// ------------------------------------------------------------------ launchers
static inline uint32_t grid_for(uint32_t n_tiles, int remap)
{
    return remap ? tiles_per_xcd(n_tiles) * kXCD : n_tiles;
}

void launch_tm(const SpmvArgs &a, hipStream_t st)
{
    const uint32_t n_tiles = ((uint32_t)a.rows + kWG - 1) / kWG;
    hipLaunchKernelGGL(spmv_tm_kernel, dim3(grid_for(n_tiles, a.remap)), dim3(kWG), 0, st,
                       a.rows, a.rp, a.ci, a.va, a.x, a.y, n_tiles, a.remap);
}

template <int G>
static void launch_wm_g(const SpmvArgs &a, hipStream_t st)
{
    constexpr uint32_t rpw = kWG / G;
    const uint32_t n_tiles = ((uint32_t)a.rows + rpw - 1) / rpw;
    hipLaunchKernelGGL(spmv_wm_kernel<G>, dim3(grid_for(n_tiles, a.remap)), dim3(kWG), 0, st,
                       a.rows, a.rp, a.ci, a.va, a.x, a.y, n_tiles, a.remap);
}

void launch_wm(const SpmvArgs &a, int G, hipStream_t st)
{
    switch (G) {
    case 2: launch_wm_g<2>(a, st); break;
    case 4: launch_wm_g<4>(a, st); break;
    case 8: launch_wm_g<8>(a, st); break;
    case 16: launch_wm_g<16>(a, st); break;
    case 32: launch_wm_g<32>(a, st); break;
    default: launch_wm_g<64>(a, st); break;
    }
}

template <int CH, bool VEC, bool NT>
static void launch_bm_v(const SpmvArgs &a, int rows_per_block, hipStream_t st)
{
    const uint32_t n_tiles = ((uint32_t)a.rows + rows_per_block - 1) / (uint32_t)rows_per_block;
    int own_shift = 0;   // rows spread over the lanes when there are fewer rows than lanes
    while ((rows_per_block << (own_shift + 1)) <= kWG) ++own_shift;
    hipLaunchKernelGGL((spmv_bm_kernel<CH, VEC, NT>), dim3(grid_for(n_tiles, a.remap)), dim3(kWG), 0, st,
                       a.rows, a.rp, a.ci, a.va, a.x, a.y, rows_per_block, own_shift, n_tiles, a.remap);
}

template <int CH>
static void launch_bm_c(const SpmvArgs &a, int rows_per_block, bool vec, hipStream_t st)
{
    if (vec) {
        if (a.nt) launch_bm_v<CH, true, true>(a, rows_per_block, st);
        else launch_bm_v<CH, true, false>(a, rows_per_block, st);
    } else {
        if (a.nt) launch_bm_v<CH, false, true>(a, rows_per_block, st);
        else launch_bm_v<CH, false, false>(a, rows_per_block, st);
    }
}

void launch_bm(const SpmvArgs &a, int rows_per_block, int chunk, bool vec, hipStream_t st)
{
    if (chunk == 4096) launch_bm_c<4096>(a, rows_per_block, vec, st);
    else launch_bm_c<2048>(a, rows_per_block, vec, st);
}

} // namespace seer
