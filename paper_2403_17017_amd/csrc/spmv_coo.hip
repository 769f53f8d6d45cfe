// Stand-alone kernels and launchers of COO,WM: the expansion of row_ptr into one row index
// per nonzero (its preprocessing) and the product; device code in spmv_bodies.hiph.
#include "spmv_bodies.hiph"

namespace seer {

__global__ __launch_bounds__(kWG) void coo_convert_kernel(int rows, const int *__restrict__ rp, int *__restrict__ crow)
{
    coo_convert_body(rows, rp, crow);
}

template <bool NT, bool RUNS>
__global__ __launch_bounds__(kWG) void spmv_coo_kernel(
    int rows, int nnz, const int *__restrict__ crow, const int *__restrict__ ci, const float *__restrict__ va,
    const float *__restrict__ x, float *__restrict__ y, int *__restrict__ carry_row,
    float *__restrict__ carry_val, uint32_t n_tiles, uint32_t n_intervals, int remap)
{
    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;
    const uint32_t w = tile * (kWG / kWave) + threadIdx.x / kWave;
    if (w >= n_intervals) return;                    // whole waves leave; the body has no barrier
    if constexpr (RUNS) coo_runs_body<NT>(rows, nnz, crow, ci, va, x, y, carry_row, carry_val, w);
    else coo_rounds_body<NT>(rows, nnz, crow, ci, va, x, y, carry_row, carry_val, w);
}

uint32_t coo_num_intervals(int rows, int nnz)
{
    if (rows <= 0) return 0;
    const uint32_t n = ((uint32_t)nnz + (uint32_t)kCooPerWave - 1u) / (uint32_t)kCooPerWave;
    return n ? n : 1u;
}

size_t coo_plan_bytes(int rows, int nnz)
{
    if (rows <= 0 || nnz < 0) return 0;
    const size_t b = ((size_t)nnz * 4 + 255) & ~(size_t)255;
    return b ? b : 256;
}

void launch_coo_convert(int rows, const int *rp, void *plan_mem, hipStream_t st)
{
    if (rows <= 0) return;
    hipLaunchKernelGGL(coo_convert_kernel, dim3(((uint32_t)rows + kWG - 1) / kWG), dim3(kWG), 0, st, rows, rp,
                       static_cast<int *>(plan_mem));
}

void launch_coo(const SpmvArgs &a, bool runs, const void *plan_mem, void *carry_ws, hipStream_t st)
{
    const uint32_t n_int = coo_num_intervals(a.rows, a.nnz);
    if (n_int == 0) return;
    const uint32_t n_tiles = (n_int + kWG / kWave - 1) / (kWG / kWave);
    const size_t one = carry_workspace_bytes(n_int) / 2;
    int *carry_row = static_cast<int *>(carry_ws);
    float *carry_val = reinterpret_cast<float *>(static_cast<char *>(carry_ws) + one);
    const int *crow = static_cast<const int *>(plan_mem);
    const dim3 grid(a.remap ? tiles_per_xcd(n_tiles) * kXCD : n_tiles);
#define SEER_COO_LAUNCH(N, R)                                                                              \
    hipLaunchKernelGGL((spmv_coo_kernel<N, R>), grid, dim3(kWG), 0, st, a.rows, a.nnz, crow, a.ci, a.va, a.x, a.y, \
                       carry_row, carry_val, n_tiles, n_int, a.remap)
    if (runs) {
        if (a.nt) SEER_COO_LAUNCH(true, true); else SEER_COO_LAUNCH(false, true);
    } else {
        if (a.nt) SEER_COO_LAUNCH(true, false); else SEER_COO_LAUNCH(false, false);
    }
#undef SEER_COO_LAUNCH
    launch_carry_fixup(a.rows, n_int, carry_row, carry_val, a.y, st);
}

} // namespace seer
