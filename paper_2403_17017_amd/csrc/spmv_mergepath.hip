// Stand-alone kernels and launchers of CSR,MP (merge path); the device code and the
// description of the algorithm are in spmv_bodies.hiph.
#include "spmv_bodies.hiph"

namespace seer {

template <int IPT, bool VEC, bool NT>
__global__ __launch_bounds__(kWG) void spmv_mp_kernel(
    int rows, int nnz, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    int *__restrict__ carry_row, float *__restrict__ carry_val, uint32_t n_tiles, int remap)
{
    __shared__ int smem[mp_lds_words<IPT>()];
    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;
    mp_body<IPT, VEC, NT>(rows, nnz, rp, ci, va, x, y, carry_row, carry_val, tile, smem);
}

__global__ __launch_bounds__(kWG) void spmv_mp_fixup_kernel(
    int rows, uint32_t n_tiles, const int *__restrict__ carry_row,
    const float *__restrict__ carry_val, float *__restrict__ y)
{
    mp_fixup_body(rows, n_tiles, carry_row, carry_val, y);
}

uint32_t mp_num_tiles(int rows, int nnz, int ipt)
{
    const uint64_t total = (uint64_t)rows + (uint64_t)nnz;
    const uint64_t T = (uint64_t)kWG * ipt;
    return (uint32_t)((total + T - 1) / T);
}

size_t mp_workspace_bytes(int rows, int nnz, int ipt)
{
    return carry_workspace_bytes(mp_num_tiles(rows, nnz, ipt));
}

void launch_carry_fixup(int rows, uint32_t n_tiles, const int *carry_row, const float *carry_val, float *y,
                        hipStream_t st)
{
    hipLaunchKernelGGL(spmv_mp_fixup_kernel, dim3((n_tiles + kWG - 1) / kWG), dim3(kWG), 0, st, rows, n_tiles,
                       carry_row, carry_val, y);
}

template <int IPT>
static void launch_mp_ipt(const SpmvArgs &a, bool vec, void *workspace, hipStream_t st)
{
    const uint32_t n_tiles = mp_num_tiles(a.rows, a.nnz, IPT);
    if (n_tiles == 0) return;
    const size_t one = carry_workspace_bytes(n_tiles) / 2;
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
    launch_carry_fixup(a.rows, n_tiles, carry_row, carry_val, a.y, st);
}

void launch_mp(const SpmvArgs &a, int ipt, bool vec, void *workspace, hipStream_t st)
{
    if (ipt == kMpIptSmall) launch_mp_ipt<kMpIptSmall>(a, vec, workspace, st);
    else launch_mp_ipt<kMpIptLarge>(a, vec, workspace, st);
}

} // namespace seer
