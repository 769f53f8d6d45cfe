// Stand-alone kernel and launcher of CSR,WO (work oriented, equal shares of nonzeros);
// the device code and the description of the split are in spmv_bodies.hiph.  The carries
// of rows cut by a chunk boundary are added to y by the same fix-up kernel as CSR,MP's.
#include "spmv_bodies.hiph"

namespace seer {

template <int CH, bool VEC, bool NT>
__global__ __launch_bounds__(kWG) void spmv_wo_kernel(
    int rows, int nnz, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const float *__restrict__ x, float *__restrict__ y,
    int *__restrict__ carry_row, float *__restrict__ carry_val, uint32_t n_tiles, int remap)
{
    __shared__ __attribute__((aligned(16))) float s_prod[bm_lds_words<CH>()];
    __shared__ uint32_t s_bounds[2];
    const uint32_t tile = tile_of_block(blockIdx.x, n_tiles, remap);
    if (tile >= n_tiles) return;
    wo_body<CH, VEC, NT>(rows, nnz, rp, ci, va, x, y, carry_row, carry_val, tile, s_prod, s_bounds);
}

uint32_t wo_num_tiles(int rows, int nnz)
{
    if (rows <= 0) return 0;
    const uint32_t ch = (uint32_t)wo_chunk_of(nnz);
    const uint32_t n = ((uint32_t)nnz + ch - 1u) / ch;
    return n ? n : 1u;   // a matrix without nonzeros still has rows to clear
}

size_t carry_workspace_bytes(uint32_t n_tiles)
{
    // carry_row then carry_val, each padded to a multiple of 256 bytes
    const size_t one = ((size_t)n_tiles * 4 + 255) & ~(size_t)255;
    return 2 * one;
}

void launch_wo(const SpmvArgs &a, bool vec, void *workspace, hipStream_t st)
{
    const uint32_t n_tiles = wo_num_tiles(a.rows, a.nnz);
    if (n_tiles == 0) return;
    const size_t one = carry_workspace_bytes(n_tiles) / 2;
    int *carry_row = static_cast<int *>(workspace);
    float *carry_val = reinterpret_cast<float *>(static_cast<char *>(workspace) + one);
    const dim3 grid(a.remap ? tiles_per_xcd(n_tiles) * kXCD : n_tiles);
#define SEER_WO_LAUNCH(C, V, N)                                                                           \
    hipLaunchKernelGGL((spmv_wo_kernel<C, V, N>), grid, dim3(kWG), 0, st, a.rows, a.nnz, a.rp, a.ci, a.va, \
                       a.x, a.y, carry_row, carry_val, n_tiles, a.remap)
#define SEER_WO_PICK(C)                                                                     \
    if (vec) {                                                                              \
        if (a.nt) SEER_WO_LAUNCH(C, true, true); else SEER_WO_LAUNCH(C, true, false);       \
    } else {                                                                                \
        if (a.nt) SEER_WO_LAUNCH(C, false, true); else SEER_WO_LAUNCH(C, false, false);     \
    }
    if (wo_chunk_of(a.nnz) == kWoChunkLarge) { SEER_WO_PICK(kWoChunkLarge) } else { SEER_WO_PICK(kWoChunk) }
#undef SEER_WO_PICK
#undef SEER_WO_LAUNCH
    launch_carry_fixup(a.rows, n_tiles, carry_row, carry_val, a.y, st);
}

} // namespace seer
