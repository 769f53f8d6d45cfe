// seer_features: the feature-collection launches (Sec. IV-A), plus two measurement
// aids (plain copy and read-only stream).  The reduction is in features_bodies.hiph.
#include "features_bodies.hiph"

namespace seer {

// Finishing (or only) launch of seer_features: the result goes into pinned host memory,
// first the statistics, then, after a system-wide fence, the sequence number.
template <bool VEC>
__global__ __launch_bounds__(kFeatWG) void features_kernel(
    int rows, const int *__restrict__ rp, const FeatPartial *__restrict__ part, uint32_t n_part,
    FeatureRaw *__restrict__ mailbox, uint64_t seq)
{
    __shared__ FeatLds s;
    features_total<VEC>(rows, rp, part, n_part, &s);
    if (threadIdx.x == 0) {
        FeatureRaw r;
        r.max_len = s.mx; r.min_len = s.mn;
        r.first = rp[0]; r.last = rp[rows];
        r.sum_sq = s.sq; r.empty = s.em; r.seq = 0;
        *mailbox = r;
        __threadfence_system();            // the statistics land before the sequence number
        *reinterpret_cast<volatile uint64_t *>(&mailbox->seq) = seq;
    }
}

// The same after a first pass, as ONE wave: it folds the partials with shuffles (no LDS, no
// barrier) and writes the result; as the workgroup of 1024 lanes above the finishing launch
// took 1.3 us longer.
__global__ __launch_bounds__(kWave) void features_wave_kernel(
    int rows, const int *__restrict__ rp, const FeatPartial *__restrict__ part, uint32_t n_part,
    FeatureRaw *__restrict__ mailbox, uint64_t seq)
{
    const int first = rp[0], last = rp[rows];
    const FeatTotals t = fold_partials_wave(part, n_part);
    if (threadIdx.x == 0) {
        FeatureRaw r;
        r.max_len = t.mx; r.min_len = t.mn;
        r.first = first; r.last = last;
        r.sum_sq = t.sq; r.empty = t.em; r.seq = 0;
        *mailbox = r;
        __threadfence_system();            // the statistics land before the sequence number
        *reinterpret_cast<volatile uint64_t *>(&mailbox->seq) = seq;
    }
}

// Plain streaming copy (measurement aid): four 16-byte loads in flight per lane and step,
// loads and stores with the streaming hint (nothing is used twice).  With one load and
// one plain store per step the same copy ran at 4.6 TB/s, below what CSR,TM streams.
__global__ __launch_bounds__(kWG) void stream_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src,
                                                          size_t n_vec)
{
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    const u4 *s = reinterpret_cast<const u4 *>(src);
    u4 *d = reinterpret_cast<u4 *>(dst);
    const size_t stride = (size_t)gridDim.x * kWG;
    size_t i = (size_t)blockIdx.x * kWG + threadIdx.x;
    for (; i + 3 * stride < n_vec; i += 4 * stride) {
        const u4 a = __builtin_nontemporal_load(s + i), b = __builtin_nontemporal_load(s + i + stride);
        const u4 c = __builtin_nontemporal_load(s + i + 2 * stride), e = __builtin_nontemporal_load(s + i + 3 * stride);
        __builtin_nontemporal_store(a, d + i);
        __builtin_nontemporal_store(b, d + i + stride);
        __builtin_nontemporal_store(c, d + i + 2 * stride);
        __builtin_nontemporal_store(e, d + i + 3 * stride);
    }
    for (; i < n_vec; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(s + i), d + i);
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

// Counts what breaks the kernels' input contract: descents in row_ptr (plus a wrong first
// or last offset) into counts[0], column indices outside [0, cols) into counts[1].  Reads
// row_ptr[0..rows] and col_idx[0..nnz-1], whatever they hold.  A well-formed matrix issues
// no atomic at all; otherwise one per wave that found something.
__global__ __launch_bounds__(kWG) void csr_check_kernel(
    int rows, int cols, int nnz, const int *__restrict__ rp, const int *__restrict__ ci,
    unsigned long long *__restrict__ counts)
{
    const size_t stride = (size_t)gridDim.x * kWG;
    const size_t first = (size_t)blockIdx.x * kWG + threadIdx.x;
    uint32_t bad_rp = 0, bad_ci = 0;
    for (size_t i = first; i < (size_t)rows; i += stride) bad_rp += rp[i + 1] < rp[i];
    if (ci)
        for (size_t k = first; k < (size_t)nnz; k += stride) bad_ci += (uint32_t)ci[k] >= (uint32_t)cols;
    if (first == 0) bad_rp += (rp[0] != 0) + (rp[rows] != nnz);
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        bad_rp += __shfl_xor(bad_rp, off);
        bad_ci += __shfl_xor(bad_ci, off);
    }
    if (threadIdx.x % kWave == 0) {
        if (bad_rp) atomicAdd(&counts[0], (unsigned long long)bad_rp);
        if (bad_ci) atomicAdd(&counts[1], (unsigned long long)bad_ci);
    }
}

void launch_csr_check(int rows, int cols, int nnz, const int *rp, const int *ci, void *counts, hipStream_t st)
{
    const size_t n = (size_t)(rows > nnz ? rows : nnz);
    const size_t want = (n + kWG * 4 - 1) / (kWG * 4);                 // about four items per lane
    const uint32_t blocks = (uint32_t)(want < 1 ? 1 : (want < 256 * 16 ? want : 256 * 16));
    hipLaunchKernelGGL(csr_check_kernel, dim3(blocks), dim3(kWG), 0, st, rows, cols, nnz, rp, ci,
                       static_cast<unsigned long long *>(counts));
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

// Gathers with streamed operands (measurement aid): sum of val[k] * x[idx[k]], indices and
// values fetched as 16-byte vectors with the streaming hint, two vectors in flight per lane
// -- the inner work of every schedule without any row handling.  With uniformly random
// indices its rate is the ceiling of a product with random columns for that size of x.
__global__ __launch_bounds__(kWG) void gather_sum_kernel(
    const v4i *__restrict__ idx, const v4f *__restrict__ val, size_t n_vec, const float *__restrict__ x,
    float *__restrict__ out)
{
    const size_t stride = (size_t)gridDim.x * kWG;
    float acc = 0.f;
    size_t i = (size_t)blockIdx.x * kWG + threadIdx.x;
    for (; i + stride < n_vec; i += 2 * stride) {
        const v4i c0 = __builtin_nontemporal_load(idx + i), c1 = __builtin_nontemporal_load(idx + i + stride);
        const v4f v0 = __builtin_nontemporal_load(val + i), v1 = __builtin_nontemporal_load(val + i + stride);
        acc += v0.x * x[c0.x] + v0.y * x[c0.y] + v0.z * x[c0.z] + v0.w * x[c0.w];
        acc += v1.x * x[c1.x] + v1.y * x[c1.y] + v1.z * x[c1.z] + v1.w * x[c1.w];
    }
    for (; i < n_vec; i += stride) {
        const v4i c = idx[i];
        const v4f v = val[i];
        acc += v.x * x[c.x] + v.y * x[c.y] + v.z * x[c.z] + v.w * x[c.w];
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    // a plain store keeps the loads alive; which wave's sum survives is irrelevant
    if (threadIdx.x % kWave == 0) out[(blockIdx.x * (kWG / kWave) + threadIdx.x / kWave) % 64] = acc;
}

void launch_gather_sum(const int *idx, const float *val, size_t n, const float *x, void *out64, hipStream_t st)
{
    const size_t n_vec = n / 4;
    if (!n_vec) return;
    const size_t want = (n_vec + kWG * 4 - 1) / (kWG * 4);
    const uint32_t blocks = (uint32_t)(want < 4096 ? want : 4096);
    hipLaunchKernelGGL(gather_sum_kernel, dim3(blocks), dim3(kWG), 0, st, reinterpret_cast<const v4i *>(idx),
                       reinterpret_cast<const v4f *>(val), n_vec, x, static_cast<float *>(out64));
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

size_t features_workspace_bytes(int rows)
{
    (void)rows;
    return (size_t)kFeatMaxParts * sizeof(FeatPartial);
}

void launch_features(int rows, const int *rp, void *workspace, FeatureRaw *mailbox_dev,
                     uint64_t seq, hipStream_t st)
{
    FeatPartial *part = static_cast<FeatPartial *>(workspace);
    const uint32_t n_part = features_num_parts(rows);
    const bool vec = (reinterpret_cast<uintptr_t>(rp) & 15u) == 0;
    if (n_part) {                                    // a first pass, then one wave
        if (vec) hipLaunchKernelGGL(features_partial_kernel<true>, dim3(n_part), dim3(kFeatPartWG), 0, st, rows, rp, part);
        else hipLaunchKernelGGL(features_partial_kernel<false>, dim3(n_part), dim3(kFeatPartWG), 0, st, rows, rp, part);
        hipLaunchKernelGGL(features_wave_kernel, dim3(1), dim3(kWave), 0, st, rows, rp, static_cast<const FeatPartial *>(part),
                           n_part, mailbox_dev, seq);
    } else if (vec) {
        hipLaunchKernelGGL(features_kernel<true>, dim3(1), dim3(kFeatWG), 0, st, rows, rp, part, n_part, mailbox_dev, seq);
    } else {
        hipLaunchKernelGGL(features_kernel<false>, dim3(1), dim3(kFeatWG), 0, st, rows, rp, part, n_part, mailbox_dev, seq);
    }
}

} // namespace seer
