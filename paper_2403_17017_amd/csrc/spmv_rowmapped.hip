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
// LDS: row_ptr segment (kBmMaxRows + 1 ints), one running sum per row, CH staged
// products, and a short list of the rows that are long inside the current chunk.
constexpr int kBmLong = 32;   // a row's overlap with a chunk above this is reduced by a wave

template <int CH, bool VEC>
__global__ __launch_bounds__(kWG) void spmv_bm_kernel(
    int rows, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    int rows_per_block, uint32_t n_tiles, int remap)
{
    static_assert(CH % (4 * kWG) == 0, "chunk must be whole float4 rounds");
    constexpr int NV = CH / (4 * kWG);
    __shared__ int s_rp[kBmMaxRows + 1];
    __shared__ float s_y[kBmMaxRows];
    __shared__ __attribute__((aligned(16))) float s_prod[CH];
    __shared__ int s_long[CH / kBmLong];
    __shared__ int s_nlong;

    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;
    const int tid = (int)threadIdx.x;
    const uint32_t r0 = tile * (uint32_t)rows_per_block;
    const int nr = (int)min((uint32_t)rows_per_block, (uint32_t)rows - r0);

    for (int i = tid; i <= nr; i += kWG) s_rp[i] = rp[r0 + i];
    for (int i = tid; i < nr; i += kWG) s_y[i] = 0.f;
    if (tid == 0) s_nlong = 0;
    __syncthreads();

    const uint32_t s = (uint32_t)s_rp[0], e = (uint32_t)s_rp[nr];
    for (uint32_t cs = s & ~3u; cs < e; cs += CH) {
        const uint32_t ce = min(cs + (uint32_t)CH, e);
        const uint32_t lo = max(cs, s);
        // ---- stage val * x[col] for [lo, ce) at s_prod[k - cs]
        int4 c[NV];
        float4 v[NV];
        bool full[NV];
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            const uint32_t k = cs + 4u * (uint32_t)(tid + kWG * m);
            full[m] = VEC && k >= lo && k + 4 <= ce;
            if (full[m]) {
                c[m] = *reinterpret_cast<const int4 *>(ci + k);
                v[m] = *reinterpret_cast<const float4 *>(va + k);
            }
        }
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            const uint32_t k = cs + 4u * (uint32_t)(tid + kWG * m);
            if (full[m]) {
                float4 p;
                p.x = v[m].x * x[c[m].x];
                p.y = v[m].y * x[c[m].y];
                p.z = v[m].z * x[c[m].z];
                p.w = v[m].w * x[c[m].w];
                *reinterpret_cast<float4 *>(s_prod + (k - cs)) = p;
            } else {
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    const uint32_t j = k + q;
                    if (j >= lo && j < ce) s_prod[j - cs] = va[j] * x[ci[j]];
                }
            }
        }
        __syncthreads();
        // ---- one lane per row: short overlaps summed in place, long ones queued
        for (int r = tid; r < nr; r += kWG) {
            const uint32_t a = max((uint32_t)s_rp[r], lo), b = min((uint32_t)s_rp[r + 1], ce);
            if (b > a) {
                if (b - a <= (uint32_t)kBmLong) {
                    float acc = 0.f;
                    for (uint32_t k = a; k < b; ++k) acc += s_prod[k - cs];
                    s_y[r] += acc;
                } else {
                    s_long[atomicAdd(&s_nlong, 1)] = r;
                }
            }
        }
        __syncthreads();
        // ---- one wave per queued row
        const int nlong = s_nlong;
        for (int q = tid / kWave; q < nlong; q += kWG / kWave) {
            const int r = s_long[q];
            const uint32_t a = max((uint32_t)s_rp[r], lo), b = min((uint32_t)s_rp[r + 1], ce);
            float acc = 0.f;
            for (uint32_t k = a + (uint32_t)(tid % kWave); k < b; k += kWave) acc += s_prod[k - cs];
            acc = group_sum<64>(acc);
            if (tid % kWave == 0) s_y[r] += acc;
        }
        __syncthreads();
        if (tid == 0) s_nlong = 0;   // next use is after the next chunk's staging barrier
    }
    for (int r = tid; r < nr; r += kWG) y[r0 + r] = s_y[r];
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

void launch_bm(const SpmvArgs &a, int rows_per_block, bool vec, hipStream_t st)
{
    const uint32_t n_tiles = ((uint32_t)a.rows + rows_per_block - 1) / (uint32_t)rows_per_block;
    const dim3 grid(grid_for(n_tiles, a.remap));
    if (vec)
        hipLaunchKernelGGL((spmv_bm_kernel<kBmChunk, true>), grid, dim3(kWG), 0, st,
                           a.rows, a.rp, a.ci, a.va, a.x, a.y, rows_per_block, n_tiles, a.remap);
    else
        hipLaunchKernelGGL((spmv_bm_kernel<kBmChunk, false>), grid, dim3(kWG), 0, st,
                           a.rows, a.rp, a.ci, a.va, a.x, a.y, rows_per_block, n_tiles, a.remap);
}

} // namespace seer
