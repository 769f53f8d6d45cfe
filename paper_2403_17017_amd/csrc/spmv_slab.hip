// CSR,S -- the column-slabbed schedule.  Not one of Table II's kernels: this build's answer
// to what bounds every schedule on a large matrix with scattered columns, the re-reading of
// x.  With x beyond one XCD's 4 MB L2 about every second gather misses and fetches a 128-byte
// line (measured on a 2 M-row power-law matrix with 8 MB of x: 7 times the algorithmic bytes
// cross the fabric, 52 of them per nonzero for x).  The preprocessing pass (Sec. IV: paid
// once, amortised over the products) stores the matrix a second time, cut by columns:
//
//   * column c belongs to slab c >> shift (2^19 columns = 2 MiB of x by default);
//   * row i becomes one virtual row per slab, virtual row s * rows + i holding the entries
//     of row i that fall into slab s (one contiguous piece of the row: its columns must
//     ascend, else the form does not apply);
//   * the entries are stored virtual row after virtual row -- all of slab 0, then slab 1 ...
//
// The product is then CSR,WO over that virtual matrix (equal shares of nonzeros, so a long
// stretch of consecutive workgroups -- one XCD's contiguous run of tiles -- gathers from
// one slab of x, which its L2 holds), into S * rows partial results, and a last pass adds
// each row's S partials in slab order.  Same power-law matrix: 382 -> 231 us per product.
// It costs S times the row handling (offsets read, partials written and read again), so
// it loses where rows are short and x fits L2 anyway; the selector decides.
#include "spmv_bodies.hiph"

namespace seer {

constexpr uint32_t kSlabLongRow = 32;       // rows beyond this are cut and copied by their whole wave
constexpr uint32_t kScanItems = 8;          // per lane of the prefix sum
constexpr uint32_t kScanTile = kWG * kScanItems;

// ---- preprocessing 1: entries per virtual row, and whether every row's columns ascend.
// cnt [S * rows + 1] is zero on entry; *descends is set if some row's columns do not ascend.
// Lane <-> row; a short row is walked entry by entry (its slab ids ascend with its columns, so
// it is a few runs), a long one is cut by binary searches for the slab boundaries, lane <-> slab.
__device__ __forceinline__ uint32_t slab_lower_bound(const int *__restrict__ ci, uint32_t a, uint32_t e, uint64_t key)
{
    while (a < e) {                          // first k in [a, e) with ci[k] >= key
        const uint32_t mid = a + (e - a) / 2u;
        if ((uint64_t)(uint32_t)ci[mid] < key) a = mid + 1u; else e = mid;
    }
    return a;
}

__global__ __launch_bounds__(kWG) void slab_count_kernel(
    int rows, int shift, uint32_t n_slabs, const int *__restrict__ rp, const int *__restrict__ ci,
    uint32_t *__restrict__ cnt, int *__restrict__ descends)
{
    const uint32_t i = blockIdx.x * kWG + threadIdx.x, lane = threadIdx.x % kWave;
    uint32_t a = 0, e = 0;
    if (i < (uint32_t)rows) {
        a = (uint32_t)rp[i];
        e = (uint32_t)rp[i + 1];
    }
    bool bad = false;
    const bool is_long = e - a > kSlabLongRow;
    if (!is_long && e > a) {
        uint32_t cur = (uint32_t)ci[a] >> shift, run = 0;
        int prev = ci[a];
        for (uint32_t k = a; k < e; ++k) {
            const int c = ci[k];
            bad |= c < prev;
            prev = c;
            const uint32_t s = (uint32_t)c >> shift;
            if (s != cur) {
                cnt[(size_t)cur * (uint32_t)rows + i] = run;
                cur = s;
                run = 0;
            }
            ++run;
        }
        cnt[(size_t)cur * (uint32_t)rows + i] = run;
    }
    uint64_t todo = __ballot(is_long);
    while (todo) {                                   // wave-uniform
        const int src = __ffsll((unsigned long long)todo) - 1;
        todo &= todo - 1;
        const uint32_t si = (uint32_t)__shfl((int)i, src), sa = (uint32_t)__shfl((int)a, src);
        const uint32_t se = (uint32_t)__shfl((int)e, src);
        for (uint32_t k = sa + 1u + lane; k < se; k += kWave) bad |= ci[k] < ci[k - 1];
        for (uint32_t s = lane; s < n_slabs; s += kWave) {
            const uint32_t lo = s == 0 ? sa : slab_lower_bound(ci, sa, se, (uint64_t)s << shift);
            const uint32_t hi = s + 1u == n_slabs ? se : slab_lower_bound(ci, sa, se, (uint64_t)(s + 1u) << shift);
            if (hi > lo) cnt[(size_t)s * (uint32_t)rows + si] = hi - lo;
        }
    }
    if (bad) *descends = 1;
}

// ---- preprocessing 2: exclusive prefix sum over n unsigned words, in place, in three kinds
// of launches: sums of tiles of 2048, the same prefix sum over those sums (recursively), and
// the tiles again with their offsets.  The total stays below 2^31 (it is nnz).
__global__ __launch_bounds__(kWG) void scan_tile_sums_kernel(const uint32_t *__restrict__ in, size_t n, uint32_t *__restrict__ sums)
{
    __shared__ uint32_t s_w[kWG / kWave];
    const size_t base = (size_t)blockIdx.x * kScanTile + (size_t)threadIdx.x * kScanItems;
    uint32_t t = 0;
#pragma unroll
    for (uint32_t j = 0; j < kScanItems; ++j)
        if (base + j < n) t += in[base + j];
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) t += (uint32_t)__shfl_xor((int)t, off);
    if (threadIdx.x % kWave == 0) s_w[threadIdx.x / kWave] = t;
    __syncthreads();
    if (threadIdx.x == 0) sums[blockIdx.x] = (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
}

__global__ __launch_bounds__(kWG) void scan_tiles_kernel(uint32_t *__restrict__ data, size_t n, const uint32_t *__restrict__ offsets /* null: one tile */)
{
    __shared__ uint32_t s_w[kWG / kWave];
    const uint32_t lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const size_t base = (size_t)blockIdx.x * kScanTile + (size_t)threadIdx.x * kScanItems;
    uint32_t v[kScanItems], t = 0;
#pragma unroll
    for (uint32_t j = 0; j < kScanItems; ++j) {
        v[j] = base + j < n ? data[base + j] : 0u;
        t += v[j];
    }
    uint32_t incl = t;                               // inclusive sum over the lanes of the wave
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)incl, off);
        if ((int)lane >= off) incl += up;
    }
    if (lane == kWave - 1) s_w[wave] = incl;
    __syncthreads();
    uint32_t before = offsets ? offsets[blockIdx.x] : 0u;
    for (uint32_t w = 0; w < wave; ++w) before += s_w[w];
    uint32_t run = before + (incl - t);
#pragma unroll
    for (uint32_t j = 0; j < kScanItems; ++j) {
        if (base + j < n) data[base + j] = run;
        run += v[j];
    }
}

static size_t scan_scratch_words(size_t n)
{
    size_t total = 0;
    while (n > kScanTile) {
        n = (n + kScanTile - 1) / kScanTile;
        total += (n + 63) & ~(size_t)63;
    }
    return total;
}

static void launch_scan_exclusive(uint32_t *data, size_t n, uint32_t *scratch, hipStream_t st)
{
    if (n <= kScanTile) {
        hipLaunchKernelGGL(scan_tiles_kernel, dim3(1), dim3(kWG), 0, st, data, n, static_cast<const uint32_t *>(nullptr));
        return;
    }
    const size_t nb = (n + kScanTile - 1) / kScanTile;
    hipLaunchKernelGGL(scan_tile_sums_kernel, dim3((uint32_t)nb), dim3(kWG), 0, st, data, n, scratch);
    launch_scan_exclusive(scratch, nb, scratch + ((nb + 63) & ~(size_t)63), st);
    hipLaunchKernelGGL(scan_tiles_kernel, dim3((uint32_t)nb), dim3(kWG), 0, st, data, n, static_cast<const uint32_t *>(scratch));
}

// ---- preprocessing 3: the entries into their places.  rp_v holds the finished offsets.
__global__ __launch_bounds__(kWG) void slab_scatter_kernel(
    int rows, int shift, uint32_t n_slabs, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const uint32_t *__restrict__ rp_v, int *__restrict__ out_ci, float *__restrict__ out_va)
{
    const uint32_t i = blockIdx.x * kWG + threadIdx.x, lane = threadIdx.x % kWave;
    uint32_t a = 0, e = 0;
    if (i < (uint32_t)rows) {
        a = (uint32_t)rp[i];
        e = (uint32_t)rp[i + 1];
    }
    const bool is_long = e - a > kSlabLongRow;
    if (!is_long && e > a) {
        uint32_t cur = 0xFFFFFFFFu, dst = 0;
        for (uint32_t k = a; k < e; ++k) {
            const int c = ci[k];
            const uint32_t s = (uint32_t)c >> shift;
            if (s != cur) {
                cur = s;
                dst = rp_v[(size_t)s * (uint32_t)rows + i];
            }
            out_ci[dst] = c;
            out_va[dst] = va[k];
            ++dst;
        }
    }
    uint64_t todo = __ballot(is_long);
    while (todo) {                                   // wave-uniform
        const int src = __ffsll((unsigned long long)todo) - 1;
        todo &= todo - 1;
        const uint32_t si = (uint32_t)__shfl((int)i, src);
        uint32_t from = (uint32_t)__shfl((int)a, src);
        for (uint32_t s = 0; s < n_slabs; ++s) {     // the row's pieces lie one after the other in it
            const size_t v = (size_t)s * (uint32_t)rows + si;
            const uint32_t d0 = rp_v[v], n = rp_v[v + 1] - d0;
            for (uint32_t j = lane; j < n; j += kWave) {
                out_ci[d0 + j] = ci[from + j];
                out_va[d0 + j] = va[from + j];
            }
            from += n;
        }
    }
}

// ---- the product's last pass: y[i] = sum over the slabs, in slab order, of the partial of
// virtual row s * rows + i.
__global__ __launch_bounds__(kWG) void slab_combine_kernel(int rows, uint32_t n_slabs, const float *__restrict__ yv, float *__restrict__ y)
{
    const uint32_t i = blockIdx.x * kWG + threadIdx.x;
    if (i >= (uint32_t)rows) return;
    float t = __builtin_nontemporal_load(yv + i);
    for (uint32_t s = 1; s < n_slabs; ++s) t += __builtin_nontemporal_load(yv + (size_t)s * (uint32_t)rows + i);
    store_y(y + i, t);
}

// ------------------------------------------------------------------ host side
static size_t pad256(size_t b) { return (b + 255) & ~(size_t)255; }

uint32_t slab_count(int rows, int cols, int shift)
{
    if (rows <= 0 || cols <= 0 || shift < 1 || shift > 30) return 0;
    const uint64_t s = ((uint64_t)cols + ((uint64_t)1 << shift) - 1) >> shift;
    if (s < 2 || s * (uint64_t)rows >= ((uint64_t)1 << 31)) return 0;
    return (uint32_t)s;
}

// plan_mem: offsets of the virtual rows [S * rows + 1], the slabbed col_idx [nnz], the slabbed
// values [nnz] (each padded to 256 bytes), then what only the preprocessing uses: the prefix
// sum's tile sums and the flag.
size_t slab_plan_bytes(int rows, int cols, int nnz, int shift)
{
    const uint32_t S = slab_count(rows, cols, shift);
    if (S == 0 || nnz < 0) return 0;
    const size_t nv = (size_t)S * (size_t)rows + 1;
    return pad256(nv * 4) + 2 * pad256((size_t)nnz * 4) + pad256(scan_scratch_words(nv) * 4) + 256;
}

// the products' scratch: the S * rows partials, then CSR,WO's carries over the virtual matrix
size_t slab_workspace_bytes(int rows, int cols, int nnz, int shift)
{
    const uint32_t S = slab_count(rows, cols, shift);
    if (S == 0) return 0;
    return pad256((size_t)S * (size_t)rows * 4) + carry_workspace_bytes(wo_num_tiles((int)(S * (uint32_t)rows), nnz));
}

int *slab_flag(void *plan_mem, int rows, int cols, int nnz, int shift)
{
    return reinterpret_cast<int *>(static_cast<char *>(plan_mem) + slab_plan_bytes(rows, cols, nnz, shift) - 256);
}

// First half of the preprocessing: counts and the check (the caller clears the counts and
// the flag before, and reads the flag after).
void launch_slab_count(int rows, int cols, int nnz, int shift, const int *rp, const int *ci, void *plan_mem, hipStream_t st)
{
    const uint32_t S = slab_count(rows, cols, shift);
    hipLaunchKernelGGL(slab_count_kernel, dim3(((uint32_t)rows + kWG - 1) / kWG), dim3(kWG), 0, st, rows, shift, S, rp, ci,
                       static_cast<uint32_t *>(plan_mem), slab_flag(plan_mem, rows, cols, nnz, shift));
}

// Second half: offsets from the counts, then the entries into their places.
void launch_slab_fill(int rows, int cols, int nnz, int shift, const int *rp, const int *ci, const float *va, void *plan_mem,
                      hipStream_t st)
{
    const uint32_t S = slab_count(rows, cols, shift);
    const size_t nv = (size_t)S * (size_t)rows + 1;
    char *base = static_cast<char *>(plan_mem);
    uint32_t *rp_v = reinterpret_cast<uint32_t *>(base);
    int *out_ci = reinterpret_cast<int *>(base + pad256(nv * 4));
    float *out_va = reinterpret_cast<float *>(base + pad256(nv * 4) + pad256((size_t)nnz * 4));
    uint32_t *scratch = reinterpret_cast<uint32_t *>(base + pad256(nv * 4) + 2 * pad256((size_t)nnz * 4));
    launch_scan_exclusive(rp_v, nv, scratch, st);
    hipLaunchKernelGGL(slab_scatter_kernel, dim3(((uint32_t)rows + kWG - 1) / kWG), dim3(kWG), 0, st, rows, shift, S, rp, ci,
                       va, static_cast<const uint32_t *>(rp_v), out_ci, out_va);
}

// The product: CSR,WO over the virtual matrix into the partials, its carry fix-up, the sum
// over the slabs.
void launch_slab(const SpmvArgs &a, uint32_t n_slabs, const void *plan_mem, void *workspace, hipStream_t st)
{
    const size_t nv = (size_t)n_slabs * (size_t)a.rows + 1;
    const char *base = static_cast<const char *>(plan_mem);
    float *yv = static_cast<float *>(workspace);
    SpmvArgs v = a;
    v.rows = (int)(n_slabs * (uint32_t)a.rows);
    v.rp = reinterpret_cast<const int *>(base);
    v.ci = reinterpret_cast<const int *>(base + pad256(nv * 4));
    v.va = reinterpret_cast<const float *>(base + pad256(nv * 4) + pad256((size_t)a.nnz * 4));
    v.y = yv;
    launch_wo(v, true, static_cast<char *>(workspace) + pad256((size_t)v.rows * 4), st);
    hipLaunchKernelGGL(slab_combine_kernel, dim3(((uint32_t)a.rows + kWG - 1) / kWG), dim3(kWG), 0, st, a.rows, n_slabs,
                       static_cast<const float *>(yv), a.y);
}

} // namespace seer
