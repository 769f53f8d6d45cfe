// Feature collection over the CSR offsets (Sec. IV-A of the Seer case study): one
// pass over row_ptr gives the longest and shortest row, the sum of squared row
// lengths and the number of empty rows.  Everything reduced here is an integer, so
// the result does not depend on the order of the reduction; the floating-point
// features are derived from these integers on the host.
//
// One launch: every workgroup reduces a grid-strided share of the rows and stores
// its partial; the workgroup that draws the last ticket folds all partials and
// writes the result straight into pinned host memory.
#include "common.hiph"
#include "launch.h"

namespace seer {

struct FeatPartial {
    int32_t max_len, min_len;
    uint64_t sum_sq, empty;
    uint64_t pad;
};
static_assert(sizeof(FeatPartial) == 32, "partials are 32 bytes apart");

constexpr uint32_t kFeatMaxBlocks = 1024;
constexpr uint32_t kFeatRowsPerBlock = kWG * 16;

// Ticket counter of the one-launch reduction.  Zero when the module is loaded and
// set back to zero by the workgroup that finishes a reduction, so back-to-back
// calls need no clearing pass.  Overlapping feature reductions on one device would
// share it and must not happen.
__device__ unsigned int g_feat_ticket = 0;

__device__ __forceinline__ void wave_fold(int32_t &mx, int32_t &mn, uint64_t &sq, uint64_t &em)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        mx = max(mx, __shfl_xor(mx, off));
        mn = min(mn, __shfl_xor(mn, off));
        sq += (uint64_t)__shfl_xor((unsigned long long)sq, off);
        em += (uint64_t)__shfl_xor((unsigned long long)em, off);
    }
}

// Folds the four statistics over the workgroup; the result is valid in thread 0.
__device__ __forceinline__ void block_fold(int32_t &mx, int32_t &mn, uint64_t &sq, uint64_t &em,
                                           FeatPartial *s_part /* LDS [4] */)
{
    wave_fold(mx, mn, sq, em);
    const uint32_t lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    __syncthreads();   // s_part may still be read from an earlier fold
    if (lane == 0) s_part[wave] = FeatPartial{mx, mn, sq, em, 0};
    __syncthreads();
    if (threadIdx.x == 0) {
        for (uint32_t w = 1; w < kWG / kWave; ++w) {
            mx = max(mx, s_part[w].max_len);
            mn = min(mn, s_part[w].min_len);
            sq += s_part[w].sum_sq;
            em += s_part[w].empty;
        }
    }
}

__global__ __launch_bounds__(kWG) void features_kernel(
    int rows, const int *__restrict__ rp, FeatPartial *__restrict__ part,
    FeatureRaw *__restrict__ mailbox, uint64_t seq)
{
    __shared__ FeatPartial s_part[kWG / kWave];
    __shared__ int s_last;
    int32_t mx = INT32_MIN, mn = INT32_MAX;
    uint64_t sq = 0, em = 0;
    const uint32_t stride = gridDim.x * kWG;
    for (uint32_t i = blockIdx.x * kWG + threadIdx.x; i < (uint32_t)rows; i += stride) {
        const int32_t len = rp[i + 1] - rp[i];
        mx = max(mx, len);
        mn = min(mn, len);
        sq += (uint64_t)((int64_t)len * (int64_t)len);
        em += len == 0;
    }
    block_fold(mx, mn, sq, em, s_part);
    if (threadIdx.x == 0) {
        part[blockIdx.x] = FeatPartial{mx, mn, sq, em, 0};
        __threadfence();                                   // partial visible device-wide ...
        const unsigned int t = atomicAdd(&g_feat_ticket, 1u);   // ... before the ticket is drawn
        s_last = (t == gridDim.x - 1);
    }
    __syncthreads();
    if (!s_last) return;

    __threadfence();   // acquire: see every other workgroup's partial
    mx = INT32_MIN; mn = INT32_MAX; sq = 0; em = 0;
    for (uint32_t b = threadIdx.x; b < gridDim.x; b += kWG) {
        const FeatPartial p = part[b];
        mx = max(mx, p.max_len);
        mn = min(mn, p.min_len);
        sq += p.sum_sq;
        em += p.empty;
    }
    block_fold(mx, mn, sq, em, s_part);
    if (threadIdx.x == 0) {
        FeatureRaw r;
        r.max_len = mx; r.min_len = mn;
        r.first = rp[0]; r.last = rp[rows];
        r.sum_sq = sq; r.empty = em; r.seq = seq;
        *mailbox = r;
        atomicExch(&g_feat_ticket, 0u);   // ready for the next call
    }
}

uint32_t features_num_blocks(int rows)
{
    if (rows <= 0) return 0;
    const uint32_t want = ((uint32_t)rows + kFeatRowsPerBlock - 1) / kFeatRowsPerBlock;
    return want < kFeatMaxBlocks ? want : kFeatMaxBlocks;
}

size_t features_workspace_bytes(int rows)
{
    (void)rows;
    return (size_t)kFeatMaxBlocks * sizeof(FeatPartial);
}

void launch_features(int rows, const int *rp, void *workspace, FeatureRaw *mailbox_dev,
                     uint64_t seq, hipStream_t st)
{
    hipLaunchKernelGGL(features_kernel, dim3(features_num_blocks(rows)), dim3(kWG), 0, st, rows, rp,
                       static_cast<FeatPartial *>(workspace), mailbox_dev, seq);
}

} // namespace seer
