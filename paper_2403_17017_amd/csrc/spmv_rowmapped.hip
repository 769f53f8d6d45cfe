// Stand-alone kernels and launchers of the row-mapped CSR SpMV schedules
// (CSR,TM / CSR,WM / CSR,BM); the device code is in spmv_bodies.hiph.
#include "spmv_bodies.hiph"

namespace seer {

template <bool SHORT, int R = 1>
__global__ __launch_bounds__(kWG) void spmv_tm_kernel(
    int rows, int nnz, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    uint32_t n_tiles, int remap)
{
    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;
    tm_body<SHORT, R>(rows, nnz, rp, ci, va, x, y, tile);
}

template <int G>
__global__ __launch_bounds__(kWG) void spmv_wm_kernel(
    int rows, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    uint32_t n_tiles, int remap)
{
    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;                 // whole workgroup leaves together
    wm_body<G>(rows, rp, ci, va, x, y, tile);
}

template <int CH, bool VEC, bool NT, bool GRP = false, int MAXR = kBmMaxRows, bool PIPE = true, bool PAD = false>
__global__ __launch_bounds__(kWG) void spmv_bm_kernel(
    int rows, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    int rows_per_block, int own_shift, uint32_t n_tiles, int remap)
{
    __shared__ __attribute__((aligned(16))) float s_prod[bm_lds_words<CH>()];
    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;
    bm_body<CH, VEC, NT, PIPE, PAD, GRP, MAXR>(rows, rp, ci, va, x, y, rows_per_block, own_shift, tile, s_prod);
}

// ------------------------------------------------------------------ launchers
static inline uint32_t grid_for(uint32_t n_tiles, int remap)
{
    return remap ? tiles_per_xcd(n_tiles) * kXCD : n_tiles;
}

bool tm_short_rows(int rows, int nnz) { return nnz >= 8 && (uint64_t)nnz <= 8ull * (uint64_t)rows; }

// Two rows per lane from 2^20 short rows on (4096 tiles of 256 rows: two full generations
// of workgroups), one otherwise.
int tm_rows_per_lane(int rows, int nnz) { return tm_short_rows(rows, nnz) && rows >= (1 << 20) ? 2 : 1; }

uint32_t tm_num_tiles(int rows, int nnz)
{
    const uint32_t per = kWG * (uint32_t)tm_rows_per_lane(rows, nnz);
    return ((uint32_t)rows + per - 1) / per;
}

void launch_tm(const SpmvArgs &a, hipStream_t st)
{
    const uint32_t n_tiles = tm_num_tiles(a.rows, a.nnz);
#define SEER_TM_LAUNCH(S, R)                                                                       \
    hipLaunchKernelGGL((spmv_tm_kernel<S, R>), dim3(grid_for(n_tiles, a.remap)), dim3(kWG), 0, st, \
                       a.rows, a.nnz, a.rp, a.ci, a.va, a.x, a.y, n_tiles, a.remap)
    if (!tm_short_rows(a.rows, a.nnz)) SEER_TM_LAUNCH(false, 1);
    else if (tm_rows_per_lane(a.rows, a.nnz) == 2) SEER_TM_LAUNCH(true, 2);
    else SEER_TM_LAUNCH(true, 1);
#undef SEER_TM_LAUNCH
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
    const int own_shift = bm_own_shift(rows_per_block);
#define SEER_BM_LAUNCH(G, M)                                                                              \
    hipLaunchKernelGGL((spmv_bm_kernel<CH, VEC, NT, G, M>), dim3(grid_for(n_tiles, a.remap)), dim3(kWG), 0, st, \
                       a.rows, a.rp, a.ci, a.va, a.x, a.y, rows_per_block, own_shift, n_tiles, a.remap)
    if (rows_per_block <= (int)kWoGroupRows) SEER_BM_LAUNCH(true, 256);   // long rows: several lanes per row
    else if (rows_per_block <= 256) SEER_BM_LAUNCH(false, 256);           // else the smallest instance that fits
    else if (rows_per_block <= 1024) SEER_BM_LAUNCH(false, 1024);
    else SEER_BM_LAUNCH(false, kBmMaxRows);
#undef SEER_BM_LAUNCH
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
