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
//   * only the virtual rows that hold entries are kept: rp_z are their offsets, and for
//     each row rp_j / p_idx list which of them are its pieces, in slab order.
//
// The product is then CSR,WO over the kept virtual rows (equal shares of nonzeros, so a long
// stretch of consecutive workgroups -- one XCD's contiguous run of tiles -- gathers from
// one slab of x, which its L2 holds), into one partial per kept virtual row, and a last pass
// adds each row's partials in slab order.  Same power-law matrix: 382 -> about 230 us per
// product.  It costs a second set of offsets and the partials' round trip, so it loses where
// rows are short and x fits L2 anyway; the selector decides.
// (A first form kept all S * rows virtual rows.  A band or a stencil leaves almost all of
// them empty, in runs of hundreds of thousands that CSR,WO hands to single workgroups: 50
// times the plain kernels' time on such matrices.)
#include "spmv_bodies.hiph"

namespace seer {

constexpr uint32_t kSlabRun = 1024;         // entries a wave takes at least: one binary search per run
constexpr uint32_t kSlabGrid = 2048;        // workgroups of the two passes over the entries
constexpr uint32_t kScanItems = 8;          // per lane of the prefix sum
constexpr uint32_t kScanTile = kWG * kScanItems;

// ---- preprocessing 1 and 3 walk the entries, not the rows: lane <-> entry, 64 at a time, every
// wave an equal contiguous run of the whole matrix, with the row of each entry read from its
// expansion crow[] (what COO,WM's conversion writes).  A "piece" is the stretch of a row that
// falls into one slab: it starts where the row or the slab id changes.  For every entry the
// first entry of its piece is the last such place at or before it -- found among the lanes by
// a ballot, carried over from step to step, and for the piece that is under way where the
// wave's run begins by one binary search in that row.
// (Lane <-> row, as the first version went, a short row is walked by one lane through cache
// lines that 63 other rows compete for, and a long one is left to one wave: 12 ms for a
// uniform matrix of 8 M rows and 1.9e8 nonzeros whose entries can be moved in under a
// millisecond, 3 ms for a 2 M-row Zipf matrix with rows of 200 000.)
__device__ __forceinline__ uint32_t slab_lower_bound(const int *__restrict__ ci, uint32_t a, uint32_t e, uint64_t key)
{
    while (a < e) {                          // first k in [a, e) with ci[k] >= key
        const uint32_t mid = a + (e - a) / 2u;
        if ((uint64_t)(uint32_t)ci[mid] < key) a = mid + 1u; else e = mid;
    }
    return a;
}

struct SlabWalk {
    uint32_t k0, k1;                         // this wave's run of entries
    uint32_t last_i, last_s;                 // row and slab of the entry before the step (none: row 0xFFFFFFFF)
    int last_c;                              // ... and its column
    uint32_t cur_start;                      // first entry of that entry's piece
};

__device__ __forceinline__ SlabWalk slab_walk_begin(
    uint32_t nnz, int shift, uint32_t n_slabs, const int *__restrict__ rp, const int *__restrict__ ci,
    const int *__restrict__ crow)
{
    const uint32_t n_waves = gridDim.x * (kWG / kWave), wv = blockIdx.x * (kWG / kWave) + threadIdx.x / kWave;
    const uint32_t per = (((nnz + n_waves - 1u) / n_waves) + kWave - 1u) & ~(uint32_t)(kWave - 1u);
    const uint64_t first = (uint64_t)wv * per;
    SlabWalk w;
    w.k0 = first < nnz ? (uint32_t)first : nnz;
    w.k1 = first + per < nnz ? (uint32_t)(first + per) : nnz;
    w.last_i = 0xFFFFFFFFu;
    w.last_s = 0;
    w.last_c = 0;
    w.cur_start = w.k0;
    if (w.k0 > 0 && w.k0 < w.k1) {
        w.last_i = (uint32_t)crow[w.k0 - 1];
        w.last_c = ci[w.k0 - 1];
        w.last_s = min((uint32_t)w.last_c >> shift, n_slabs - 1u);
        w.cur_start = slab_lower_bound(ci, (uint32_t)rp[w.last_i], w.k0, (uint64_t)w.last_s << shift);
    }
    return w;
}

// One step: the lane's entry (row i, column c, slab s), whether it is valid, and the first
// entry of its piece.  Updates the carry.  All lanes of the wave call it together.
__device__ __forceinline__ uint32_t slab_walk_step(
    SlabWalk &w, uint32_t base, uint32_t lane, int shift, uint32_t n_slabs, const int *__restrict__ ci,
    const int *__restrict__ crow, bool &valid, uint32_t &i, int &c, uint32_t &s, bool &descends)
{
    const uint32_t k = base + lane;
    valid = k < w.k1;
    i = valid ? (uint32_t)crow[k] : 0u;
    c = valid ? ci[k] : 0;
    s = min((uint32_t)c >> shift, n_slabs - 1u);
    uint32_t pi = (uint32_t)__shfl_up((int)i, 1), ps = (uint32_t)__shfl_up((int)s, 1);
    int pc = __shfl_up(c, 1);
    if (lane == 0) { pi = w.last_i; ps = w.last_s; pc = w.last_c; }
    const bool starts = valid && (i != pi || s != ps);
    descends = valid && i == pi && c < pc;
    const uint64_t mask = __ballot(starts);
    const uint64_t upto = mask & (lane == kWave - 1 ? ~0ull : ((1ull << (lane + 1u)) - 1ull));
    const uint32_t mine = upto ? base + 63u - (uint32_t)__clzll((long long)upto) : w.cur_start;
    if (mask) w.cur_start = base + 63u - (uint32_t)__clzll((long long)mask);
    const int last = (int)min(w.k1 - base, (uint32_t)kWave) - 1;
    w.last_i = (uint32_t)__shfl((int)i, last);
    w.last_s = (uint32_t)__shfl((int)s, last);
    w.last_c = __shfl(c, last);
    return mine;
}

// preprocessing 1: entries per virtual row (cnt [S * rows + 1], zero on entry), written by the
// last entry of each piece; *flag is set if some row's columns do not ascend or lie outside
// the matrix (then the form is refused instead of written out of bounds).
__global__ __launch_bounds__(kWG) void slab_count_kernel(
    int rows, int cols, uint32_t nnz, int shift, uint32_t n_slabs, const int *__restrict__ rp,
    const int *__restrict__ ci, const int *__restrict__ crow, uint32_t *__restrict__ cnt, int *__restrict__ flag)
{
    const uint32_t lane = threadIdx.x % kWave;
    SlabWalk w = slab_walk_begin(nnz, shift, n_slabs, rp, ci, crow);
    bool bad = false;
    for (uint32_t base = w.k0; base < w.k1; base += kWave) {       // wave-uniform
        bool valid, desc;
        uint32_t i, s;
        int c;
        const uint32_t mine = slab_walk_step(w, base, lane, shift, n_slabs, ci, crow, valid, i, c, s, desc);
        bad |= desc || (valid && (uint32_t)c >= (uint32_t)cols);
        if (!valid) continue;
        const uint32_t k = base + lane;
        bool ends = k + 1u == nnz;
        if (!ends) {
            const uint32_t ni = (uint32_t)crow[k + 1u];
            const uint32_t ns = min((uint32_t)ci[k + 1u] >> shift, n_slabs - 1u);
            ends = ni != i || ns != s;
        }
        if (ends) cnt[(size_t)s * (uint32_t)rows + i] = k + 1u - mine;
    }
    if (bad) *flag = 1;
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

// ---- preprocessing 3: the entries into their places.  rp_v holds the finished offsets: an
// entry goes to (start of its virtual row) + (its distance from the first entry of its piece).
__global__ __launch_bounds__(kWG) void slab_scatter_kernel(
    int rows, uint32_t nnz, int shift, uint32_t n_slabs, const int *__restrict__ rp, const int *__restrict__ ci,
    const float *__restrict__ va, const int *__restrict__ crow, const uint32_t *__restrict__ rp_v,
    int *__restrict__ out_ci, float *__restrict__ out_va)
{
    const uint32_t lane = threadIdx.x % kWave;
    SlabWalk w = slab_walk_begin(nnz, shift, n_slabs, rp, ci, crow);
    for (uint32_t base = w.k0; base < w.k1; base += kWave) {       // wave-uniform
        bool valid, desc;
        uint32_t i, s;
        int c;
        const uint32_t mine = slab_walk_step(w, base, lane, shift, n_slabs, ci, crow, valid, i, c, s, desc);
        if (!valid) continue;
        const uint32_t k = base + lane;
        const uint32_t dst = rp_v[(size_t)s * (uint32_t)rows + i] + (k - mine);
        out_ci[dst] = c;
        out_va[dst] = va[k];
    }
}

// ---- preprocessing 4 to 6: which virtual rows hold entries.
// Pieces per row (cnt still holds the counts): lane <-> row.
__global__ __launch_bounds__(kWG) void slab_row_pieces_kernel(int rows, uint32_t n_slabs, const uint32_t *__restrict__ cnt,
                                                              uint32_t *__restrict__ pieces /* [rows + 1], last stays 0 */)
{
    const uint32_t i = blockIdx.x * kWG + threadIdx.x;
    if (i >= (uint32_t)rows) return;
    uint32_t n = 0;
    for (uint32_t s = 0; s < n_slabs; ++s) n += cnt[(size_t)s * (uint32_t)rows + i] != 0u;
    pieces[i] = n;
}

// 1 for a virtual row with entries, else 0 (then prefix-summed into the kept rows' numbers).
__global__ __launch_bounds__(kWG) void slab_flags_kernel(size_t nv, const uint32_t *__restrict__ cnt, uint32_t *__restrict__ keep)
{
    const size_t stride = (size_t)gridDim.x * kWG;
    for (size_t v = (size_t)blockIdx.x * kWG + threadIdx.x; v < nv; v += stride) keep[v] = v + 1 < nv && cnt[v] != 0u;
}

// With rp_v (offsets of all virtual rows) and num_v (number of kept rows before each) done:
// the kept rows' offsets rp_z, and per row the numbers of its pieces, in slab order.
__global__ __launch_bounds__(kWG) void slab_compact_kernel(
    int rows, uint32_t n_slabs, const uint32_t *__restrict__ rp_v, const uint32_t *__restrict__ num_v,
    const uint32_t *__restrict__ rp_j, uint32_t n_kept, uint32_t nnz, uint32_t *__restrict__ rp_z, uint32_t *__restrict__ p_idx)
{
    const uint32_t i = blockIdx.x * kWG + threadIdx.x;
    if (i == 0) rp_z[n_kept] = nnz;
    if (i >= (uint32_t)rows) return;
    uint32_t t = rp_j[i];
    for (uint32_t s = 0; s < n_slabs; ++s) {
        const size_t v = (size_t)s * (uint32_t)rows + i;
        const uint32_t a = rp_v[v];
        if (rp_v[v + 1] != a) {
            const uint32_t j = num_v[v];
            rp_z[j] = a;
            p_idx[t++] = j;
        }
    }
}

// ---- the product's last pass: y[i] = sum of the partials of row i's pieces, in slab order.
__global__ __launch_bounds__(kWG) void slab_combine_kernel(
    int rows, const uint32_t *__restrict__ rp_j, const uint32_t *__restrict__ p_idx, const float *__restrict__ yz,
    float *__restrict__ y)
{
    const uint32_t i = blockIdx.x * kWG + threadIdx.x;
    if (i >= (uint32_t)rows) return;
    const uint32_t a = __builtin_nontemporal_load(rp_j + i), e = __builtin_nontemporal_load(rp_j + i + 1);
    float t = 0.f;
    if (e - a <= 4u) {                               // the usual case: fetched together
        float p[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q)
            if (a + q < e) p[q] = yz[__builtin_nontemporal_load(p_idx + a + q)];
        t = ((p[0] + p[1]) + p[2]) + p[3];
    } else {
        for (uint32_t k = a; k < e; ++k) t += yz[__builtin_nontemporal_load(p_idx + k)];
    }
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

// Where things lie in plan_mem.  What the products read comes first, sized for the most
// virtual rows that can hold entries (min(nnz, S * rows)), so that the layout follows from the
// sizes alone: rp_z, p_idx, rp_j, the slabbed col_idx, the slabbed values; then what only the
// preprocessing uses: the offsets and the kept-row numbers of all S * rows virtual rows, the
// row of every entry, the prefix
// sums' tile sums, the flag.
struct SlabLayout {
    size_t nv, max_kept;
    size_t rp_z, p_idx, rp_j, ci, va, rp_v, num_v, crow, scan, flag, total;
};
static SlabLayout slab_layout(uint32_t S, int rows, int nnz)
{
    SlabLayout L;
    L.nv = (size_t)S * (size_t)rows + 1;
    L.max_kept = (size_t)nnz < L.nv - 1 ? (size_t)nnz : L.nv - 1;
    size_t o = 0;
    L.rp_z = o;  o += pad256((L.max_kept + 1) * 4);
    L.p_idx = o; o += pad256(L.max_kept * 4 + 4);
    L.rp_j = o;  o += pad256(((size_t)rows + 1) * 4);
    L.ci = o;    o += pad256((size_t)nnz * 4 + 4);
    L.va = o;    o += pad256((size_t)nnz * 4 + 4);
    L.rp_v = o;  o += pad256(L.nv * 4);
    L.num_v = o; o += pad256(L.nv * 4);
    L.crow = o;  o += pad256((size_t)nnz * 4 + 4);
    L.scan = o;  o += pad256(scan_scratch_words(L.nv) * 4 + 4);
    L.flag = o;  o += 256;
    L.total = o;
    return L;
}

size_t slab_plan_bytes(int rows, int cols, int nnz, int shift)
{
    const uint32_t S = slab_count(rows, cols, shift);
    if (S == 0 || nnz < 0) return 0;
    return slab_layout(S, rows, nnz).total;
}

// the products' scratch: one partial per kept virtual row, then CSR,WO's carries over them
size_t slab_workspace_bytes(uint32_t n_kept, int nnz)
{
    return pad256((size_t)n_kept * 4 + 4) + carry_workspace_bytes(wo_num_tiles((int)n_kept, nnz));
}

int *slab_flag(void *plan_mem, int rows, int cols, int nnz, int shift)
{
    return reinterpret_cast<int *>(static_cast<char *>(plan_mem) + slab_layout(slab_count(rows, cols, shift), rows, nnz).flag);
}

const uint32_t *slab_kept_count(const void *plan_mem, int rows, int cols, int nnz, int shift)
{
    // rp_j[rows] = the number of kept virtual rows, once launch_slab_count has run
    return reinterpret_cast<const uint32_t *>(static_cast<const char *>(plan_mem) +
                                              slab_layout(slab_count(rows, cols, shift), rows, nnz).rp_j) + rows;
}

// no more workgroups than runs of kSlabRun entries
static uint32_t slab_entry_grid(int nnz)
{
    const uint32_t most = (uint32_t)nnz / kSlabRun / (kWG / kWave) + 1u;
    return most < kSlabGrid ? most : kSlabGrid;
}

// First half of the preprocessing: the row of every entry, entries per virtual row with the
// check of the columns, and the pieces per row prefix-summed into rp_j.  Clears what it needs cleared.  The
// caller then waits, reads the flag and rp_j[rows].
void launch_slab_count(int rows, int cols, int nnz, int shift, const int *rp, const int *ci, void *plan_mem, hipStream_t st)
{
    const uint32_t S = slab_count(rows, cols, shift);
    const SlabLayout L = slab_layout(S, rows, nnz);
    char *base = static_cast<char *>(plan_mem);
    uint32_t *cnt = reinterpret_cast<uint32_t *>(base + L.rp_v);
    uint32_t *rp_j = reinterpret_cast<uint32_t *>(base + L.rp_j);
    (void)hipMemsetAsync(cnt, 0, L.nv * 4, st);
    (void)hipMemsetAsync(base + L.flag, 0, sizeof(int), st);
    (void)hipMemsetAsync(rp_j + rows, 0, 4, st);
    int *crow = reinterpret_cast<int *>(base + L.crow);
    launch_coo_convert(rows, rp, crow, st);
    hipLaunchKernelGGL(slab_count_kernel, dim3(slab_entry_grid(nnz)), dim3(kWG), 0, st, rows, cols, (uint32_t)nnz, shift, S,
                       rp, ci, static_cast<const int *>(crow), cnt, reinterpret_cast<int *>(base + L.flag));
    const dim3 by_rows(((uint32_t)rows + kWG - 1) / kWG);
    hipLaunchKernelGGL(slab_row_pieces_kernel, by_rows, dim3(kWG), 0, st, rows, S, static_cast<const uint32_t *>(cnt), rp_j);
    launch_scan_exclusive(rp_j, (size_t)rows + 1, reinterpret_cast<uint32_t *>(base + L.scan), st);
}

// Second half: the numbers of the kept rows, the offsets of all virtual rows, the kept rows'
// offsets and each row's list of pieces, then the entries into their places.
void launch_slab_fill(int rows, int cols, int nnz, int shift, uint32_t n_kept, const int *rp, const int *ci, const float *va,
                      void *plan_mem, hipStream_t st)
{
    const uint32_t S = slab_count(rows, cols, shift);
    const SlabLayout L = slab_layout(S, rows, nnz);
    char *base = static_cast<char *>(plan_mem);
    uint32_t *rp_v = reinterpret_cast<uint32_t *>(base + L.rp_v), *num_v = reinterpret_cast<uint32_t *>(base + L.num_v);
    uint32_t *scratch = reinterpret_cast<uint32_t *>(base + L.scan);
    const size_t want = (L.nv + kWG * 8 - 1) / (kWG * 8);
    hipLaunchKernelGGL(slab_flags_kernel, dim3((uint32_t)(want < 65536 ? want : 65536)), dim3(kWG), 0, st, L.nv,
                       static_cast<const uint32_t *>(rp_v), num_v);
    launch_scan_exclusive(num_v, L.nv, scratch, st);
    launch_scan_exclusive(rp_v, L.nv, scratch, st);
    const dim3 by_rows(((uint32_t)rows + kWG - 1) / kWG);
    hipLaunchKernelGGL(slab_compact_kernel, by_rows, dim3(kWG), 0, st, rows, S, static_cast<const uint32_t *>(rp_v),
                       static_cast<const uint32_t *>(num_v), reinterpret_cast<const uint32_t *>(base + L.rp_j), n_kept,
                       (uint32_t)nnz, reinterpret_cast<uint32_t *>(base + L.rp_z), reinterpret_cast<uint32_t *>(base + L.p_idx));
    hipLaunchKernelGGL(slab_scatter_kernel, dim3(slab_entry_grid(nnz)), dim3(kWG), 0, st, rows, (uint32_t)nnz, shift, S, rp,
                       ci, va, reinterpret_cast<const int *>(base + L.crow), static_cast<const uint32_t *>(rp_v),
                       reinterpret_cast<int *>(base + L.ci), reinterpret_cast<float *>(base + L.va));
}

// The product: CSR,WO over the kept virtual rows into their partials, its carry fix-up, the
// sum over each row's pieces.
void launch_slab(const SpmvArgs &a, uint32_t n_slabs, uint32_t n_kept, const void *plan_mem, void *workspace, hipStream_t st)
{
    const SlabLayout L = slab_layout(n_slabs, a.rows, a.nnz);
    const char *base = static_cast<const char *>(plan_mem);
    float *yz = static_cast<float *>(workspace);
    if (n_kept) {
        SpmvArgs v = a;
        v.rows = (int)n_kept;
        v.rp = reinterpret_cast<const int *>(base + L.rp_z);
        v.ci = reinterpret_cast<const int *>(base + L.ci);
        v.va = reinterpret_cast<const float *>(base + L.va);
        v.y = yz;
        launch_wo(v, true, static_cast<char *>(workspace) + pad256((size_t)n_kept * 4 + 4), st);
    }
    hipLaunchKernelGGL(slab_combine_kernel, dim3(((uint32_t)a.rows + kWG - 1) / kWG), dim3(kWG), 0, st, a.rows,
                       reinterpret_cast<const uint32_t *>(base + L.rp_j), reinterpret_cast<const uint32_t *>(base + L.p_idx),
                       static_cast<const float *>(yz), a.y);
}

} // namespace seer
