// Stand-alone kernels and launchers of CSR,A (adaptive: row blocks found in a
// preprocessing pass); device code and description are in spmv_bodies.hiph.
#include "spmv_bodies.hiph"

namespace seer {

__global__ __launch_bounds__(kWG) void adaptive_plan_kernel(
    int rows, int nnz, const int *__restrict__ rp, int2 *__restrict__ plan, uint32_t n_tiles,
    int *__restrict__ split_flag)
{
    adaptive_plan_body<kAdaptChunk>(rows, nnz, rp, plan, n_tiles, split_flag);
}

template <bool VEC, bool NT>
__global__ __launch_bounds__(kWG) void spmv_adaptive_kernel(
    int rows, const int *__restrict__ rp, const int *__restrict__ ci, const float *__restrict__ va,
    const float *__restrict__ x, float *__restrict__ y, const int2 *__restrict__ plan,
    int *__restrict__ carry_row, float *__restrict__ carry_val, uint32_t n_tiles, int remap)
{
    __shared__ __attribute__((aligned(16))) float s_prod[2 * kAdaptChunk];
    __shared__ float s_red[4];
    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;
    adaptive_body<kAdaptChunk, VEC, NT>(rows, rp, ci, va, x, y, plan, carry_row, carry_val, tile, s_prod, s_red);
}

uint32_t adaptive_num_tiles(int rows, int nnz)
{
    if (rows <= 0) return 0;
    const uint32_t n = ((uint32_t)nnz + (uint32_t)kAdaptChunk - 1u) / (uint32_t)kAdaptChunk;
    return n ? n : 1u;
}

// plan entries (n + 1 pairs), padded to 256 bytes, then one word: "some row is split"
size_t adaptive_plan_bytes(int rows, int nnz)
{
    const size_t n = adaptive_num_tiles(rows, nnz);
    return (((n + 1) * sizeof(int2) + 255) & ~(size_t)255) + 256;
}

int *adaptive_split_flag(void *plan_mem, int rows, int nnz)
{
    return reinterpret_cast<int *>(static_cast<char *>(plan_mem) + adaptive_plan_bytes(rows, nnz) - 256);
}

void launch_adaptive_plan(int rows, int nnz, const int *rp, void *plan_mem, bool want_flag, hipStream_t st)
{
    const uint32_t n_tiles = adaptive_num_tiles(rows, nnz);
    if (n_tiles == 0) return;
    hipLaunchKernelGGL(adaptive_plan_kernel, dim3(((uint32_t)rows + kWG - 1) / kWG), dim3(kWG), 0, st, rows, nnz, rp,
                       static_cast<int2 *>(plan_mem), n_tiles,
                       want_flag ? adaptive_split_flag(plan_mem, rows, nnz) : nullptr);
}

void launch_adaptive(const SpmvArgs &a, bool vec, const void *plan_mem, void *carry_ws, hipStream_t st)
{
    const uint32_t n_tiles = adaptive_num_tiles(a.rows, a.nnz);
    if (n_tiles == 0) return;
    const size_t one = carry_workspace_bytes(n_tiles) / 2;
    int *carry_row = static_cast<int *>(carry_ws);
    float *carry_val = carry_ws ? reinterpret_cast<float *>(static_cast<char *>(carry_ws) + one) : nullptr;
    const int2 *plan = static_cast<const int2 *>(plan_mem);
    const dim3 grid(a.remap ? tiles_per_xcd(n_tiles) * kXCD : n_tiles);
#define SEER_A_LAUNCH(V, N)                                                                            \
    hipLaunchKernelGGL((spmv_adaptive_kernel<V, N>), grid, dim3(kWG), 0, st, a.rows, a.rp, a.ci, a.va, a.x, \
                       a.y, plan, carry_row, carry_val, n_tiles, a.remap)
    if (vec) {
        if (a.nt) SEER_A_LAUNCH(true, true); else SEER_A_LAUNCH(true, false);
    } else {
        if (a.nt) SEER_A_LAUNCH(false, true); else SEER_A_LAUNCH(false, false);
    }
#undef SEER_A_LAUNCH
    if (carry_ws) launch_carry_fixup(a.rows, n_tiles, carry_row, carry_val, a.y, st);
}

} // namespace seer
