// Stand-alone kernels and launchers of ELL,TM: the conversion from CSR (its preprocessing)
// and the product; device code and layout are described in spmv_bodies.hiph.
#include "spmv_bodies.hiph"

namespace seer {

__global__ __launch_bounds__(kWG) void ell_convert_kernel(
    int rows, uint32_t rows_pad, uint32_t width, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, int *__restrict__ ec, float *__restrict__ ev)
{
    ell_convert_body(rows, rows_pad, width, rp, ci, va, ec, ev);
}

template <bool NT>
__global__ __launch_bounds__(kWG) void spmv_ell_kernel(
    int rows, uint32_t rows_pad, uint32_t width, const int *__restrict__ ec, const float *__restrict__ ev,
    const float *__restrict__ x, float *__restrict__ y, uint32_t n_tiles, int remap)
{
    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;
    ell_body<NT>(rows, rows_pad, width, ec, ev, x, y, tile);
}

uint32_t ell_rows_pad(int rows) { return ((uint32_t)rows + kEllRowMultiple - 1) / kEllRowMultiple * kEllRowMultiple; }

// columns then values, each rows_pad * width words; 0 if the arrays cannot be indexed
size_t ell_plan_bytes(int rows, int width)
{
    if (rows <= 0 || width < 0) return 0;
    const uint64_t words = (uint64_t)ell_rows_pad(rows) * (uint64_t)width;
    if (words >= (1ull << 31)) return 0;
    const size_t one = ((size_t)words * 4 + 255) & ~(size_t)255;
    return one ? 2 * one : 256;
}

static float *ell_values(void *plan_mem, int rows, int width)
{
    return reinterpret_cast<float *>(static_cast<char *>(plan_mem) + ell_plan_bytes(rows, width) / 2);
}

void launch_ell_convert(int rows, int width, const int *rp, const int *ci, const float *va, void *plan_mem,
                        hipStream_t st)
{
    if (rows <= 0 || width <= 0) return;
    const uint32_t rows_pad = ell_rows_pad(rows);
    hipLaunchKernelGGL(ell_convert_kernel, dim3((rows_pad + kWG - 1) / kWG), dim3(kWG), 0, st, rows, rows_pad,
                       (uint32_t)width, rp, ci, va, static_cast<int *>(plan_mem), ell_values(plan_mem, rows, width));
}

void launch_ell(const SpmvArgs &a, int width, const void *plan_mem, hipStream_t st)
{
    if (a.rows <= 0) return;
    const uint32_t rows_pad = ell_rows_pad(a.rows), n_tiles = ((uint32_t)a.rows + kWG - 1) / kWG;
    const int *ec = static_cast<const int *>(plan_mem);
    const float *ev = ell_values(const_cast<void *>(plan_mem), a.rows, width);
    const dim3 grid(a.remap ? tiles_per_xcd(n_tiles) * kXCD : n_tiles);
    if (a.nt)
        hipLaunchKernelGGL(spmv_ell_kernel<true>, grid, dim3(kWG), 0, st, a.rows, rows_pad, (uint32_t)width, ec, ev,
                           a.x, a.y, n_tiles, a.remap);
    else
        hipLaunchKernelGGL(spmv_ell_kernel<false>, grid, dim3(kWG), 0, st, a.rows, rows_pad, (uint32_t)width, ec, ev,
                           a.x, a.y, n_tiles, a.remap);
}

} // namespace seer
