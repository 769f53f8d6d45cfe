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

// Few, large workgroups: every workgroup ends with one atomic on a single counter,
// and those are served one after the other (about 25 ns each), so their number,
// not the streaming of row_ptr, would otherwise set the kernel's duration.
constexpr uint32_t kFeatWG = 1024;
constexpr uint32_t kFeatWaves = kFeatWG / kWave;
constexpr uint32_t kFeatMaxBlocks = 64;
constexpr uint32_t kFeatRowsPerBlock = kFeatWG * 8;   // two 16-byte loads of row_ptr per lane

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
                                           FeatPartial *s_part /* LDS [kFeatWaves] */)
{
    wave_fold(mx, mn, sq, em);
    const uint32_t lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    __syncthreads();   // s_part may still be read from an earlier fold
    if (lane == 0) s_part[wave] = FeatPartial{mx, mn, sq, em, 0};
    __syncthreads();
    if (threadIdx.x == 0) {
        for (uint32_t w = 1; w < kFeatWaves; ++w) {
            mx = max(mx, s_part[w].max_len);
            mn = min(mn, s_part[w].min_len);
            sq += s_part[w].sum_sq;
            em += s_part[w].empty;
        }
    }
}

__device__ __forceinline__ void take_row(int32_t len, int32_t &mx, int32_t &mn, uint64_t &sq, uint64_t &em)
{
    mx = max(mx, len);
    mn = min(mn, len);
    sq += (uint64_t)((int64_t)len * (int64_t)len);
    em += len == 0;
}

// VEC: row_ptr is 16-byte aligned; lane handles rows 4q .. 4q+3 from one 16-byte load
// plus the first offset of the next quad.  row_ptr is loaded with plain (temporal)
// loads on purpose: the SpMV that follows reads it again.
template <bool VEC>
__global__ __launch_bounds__(kFeatWG) void features_kernel(
    int rows, const int *__restrict__ rp, FeatPartial *__restrict__ part,
    FeatureRaw *__restrict__ mailbox, uint64_t seq)
{
    __shared__ FeatPartial s_part[kFeatWaves];
    __shared__ int s_last;
    int32_t mx = INT32_MIN, mn = INT32_MAX;
    uint64_t sq = 0, em = 0;
    const uint32_t stride = gridDim.x * kFeatWG;
    if constexpr (VEC) {
        const uint32_t n_quads = (uint32_t)rows / 4u;
        uint32_t q = blockIdx.x * kFeatWG + threadIdx.x;
        for (; q + stride < n_quads; q += 2 * stride) {      // two independent quads in flight
            const v4i v = *reinterpret_cast<const v4i *>(rp + 4u * q);
            const v4i w = *reinterpret_cast<const v4i *>(rp + 4u * (q + stride));
            const int32_t vn = rp[4u * q + 4u], wn = rp[4u * (q + stride) + 4u];
            take_row(v.y - v.x, mx, mn, sq, em);
            take_row(v.z - v.y, mx, mn, sq, em);
            take_row(v.w - v.z, mx, mn, sq, em);
            take_row(vn - v.w, mx, mn, sq, em);
            take_row(w.y - w.x, mx, mn, sq, em);
            take_row(w.z - w.y, mx, mn, sq, em);
            take_row(w.w - w.z, mx, mn, sq, em);
            take_row(wn - w.w, mx, mn, sq, em);
        }
        if (q < n_quads) {
            const v4i v = *reinterpret_cast<const v4i *>(rp + 4u * q);
            const int32_t vn = rp[4u * q + 4u];
            take_row(v.y - v.x, mx, mn, sq, em);
            take_row(v.z - v.y, mx, mn, sq, em);
            take_row(v.w - v.z, mx, mn, sq, em);
            take_row(vn - v.w, mx, mn, sq, em);
        }
        if (blockIdx.x == 0 && threadIdx.x < ((uint32_t)rows & 3u)) {   // the last 0..3 rows
            const uint32_t i = n_quads * 4u + threadIdx.x;
            take_row(rp[i + 1] - rp[i], mx, mn, sq, em);
        }
    } else {
        for (uint32_t i = blockIdx.x * kFeatWG + threadIdx.x; i < (uint32_t)rows; i += stride)
            take_row(rp[i + 1] - rp[i], mx, mn, sq, em);
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
    for (uint32_t b = threadIdx.x; b < gridDim.x; b += kFeatWG) {
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
        r.sum_sq = sq; r.empty = em; r.seq = 0;
        *mailbox = r;
        __threadfence_system();            // the statistics land before the sequence number
        *reinterpret_cast<volatile uint64_t *>(&mailbox->seq) = seq;
        atomicExch(&g_feat_ticket, 0u);    // ready for the next call
    }
}

// Plain streaming copy (measurement aid): one 16-byte load and store per lane and step.
__global__ __launch_bounds__(kWG) void stream_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src,
                                                          size_t n_vec)
{
    const size_t stride = (size_t)gridDim.x * kWG;
    for (size_t i = (size_t)blockIdx.x * kWG + threadIdx.x; i < n_vec; i += stride) dst[i] = src[i];
}

__global__ void stream_copy_tail_kernel(uint32_t *__restrict__ dst, const uint32_t *__restrict__ src, size_t from,
                                        size_t n_words)
{
    const size_t i = from + threadIdx.x;
    if (i < n_words) dst[i] = src[i];
}

// Read-only stream (measurement aid): every lane adds up its share, one word per
// workgroup is written.
__global__ __launch_bounds__(kWG) void stream_sum_kernel(const uint4 *__restrict__ src, size_t n_vec,
                                                         uint32_t *__restrict__ out)
{
    const size_t stride = (size_t)gridDim.x * kWG;
    uint32_t acc = 0;
    for (size_t i = (size_t)blockIdx.x * kWG + threadIdx.x; i < n_vec; i += stride) {
        const uint4 v = src[i];
        acc += v.x ^ v.y ^ v.z ^ v.w;
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    // a plain store keeps the loads alive; which wave's checksum survives is irrelevant
    if (threadIdx.x % kWave == 0) out[(blockIdx.x * (kWG / kWave) + threadIdx.x / kWave) % 64] = acc;
}

void launch_stream_sum(const void *src, size_t n_words, void *out64, hipStream_t st)
{
    const size_t n_vec = n_words / 4;
    if (!n_vec) return;
    const size_t want = (n_vec + kWG * 4 - 1) / (kWG * 4);
    const uint32_t blocks = (uint32_t)(want < 256 * 32 ? want : 256 * 32);
    hipLaunchKernelGGL(stream_sum_kernel, dim3(blocks), dim3(kWG), 0, st, static_cast<const uint4 *>(src), n_vec,
                       static_cast<uint32_t *>(out64));
}

void launch_stream_copy(void *dst, const void *src, size_t n_words, hipStream_t st)
{
    const size_t n_vec = n_words / 4;
    if (n_vec) {
        const size_t want = (n_vec + kWG * 4 - 1) / (kWG * 4);
        const uint32_t blocks = (uint32_t)(want < 256 * 32 ? want : 256 * 32);
        hipLaunchKernelGGL(stream_copy_kernel, dim3(blocks), dim3(kWG), 0, st, static_cast<uint4 *>(dst),
                           static_cast<const uint4 *>(src), n_vec);
    }
    if (n_words % 4)
        hipLaunchKernelGGL(stream_copy_tail_kernel, dim3(1), dim3(4), 0, st, static_cast<uint32_t *>(dst),
                           static_cast<const uint32_t *>(src), n_vec * 4, n_words);
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
    if ((reinterpret_cast<uintptr_t>(rp) & 15u) == 0)
        hipLaunchKernelGGL(features_kernel<true>, dim3(features_num_blocks(rows)), dim3(kFeatWG), 0, st, rows, rp,
                           static_cast<FeatPartial *>(workspace), mailbox_dev, seq);
    else
        hipLaunchKernelGGL(features_kernel<false>, dim3(features_num_blocks(rows)), dim3(kFeatWG), 0, st, rows, rp,
                           static_cast<FeatPartial *>(workspace), mailbox_dev, seq);
}

} // namespace seer
