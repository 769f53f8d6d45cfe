// C ABI of the library: argument checks, launch heuristics that need only the
// trivially known sizes (rows, nnz), the host-side feature derivation and the
// decision-tree walk.  No device memory is allocated here.
#include "../../include/seer.h"
#include "launch.h"
// The trained models in the form they are deployed in (Sec. III-D): nested if/else code
// generated from the fitted trees; what the entry points use when the caller passes no model.
#include "../selector_model_generated.h"

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdlib>
#include <cstring>
#include <mutex>

using namespace seer;

// Scratch of seer_spmv_auto_static, the entry point for callers that cannot allocate: feature
// partials, the selection record and the tile carry-outs of the asynchronous path.  Every
// GPU the library runs on holds its own copy of this array until the process ends.  In host
// code the name below is only a handle for hipGetSymbolAddress; kernels get the address
// that call returns.
constexpr size_t kStaticScratchBytes = SEER_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};     // device address of `scratch` on each device, once looked up

std::atomic<int> g_last_hip_error{0};

// Tuning hooks (negative = choose automatically).
std::atomic<int> g_tune_wm_lanes{-1};
std::atomic<int> g_tune_bm_rows{-1};
std::atomic<int> g_tune_bm_chunk{-1};
std::atomic<int> g_tune_mp_ipt{-1};
std::atomic<int> g_tune_fused_rows{-1};
std::atomic<int> g_tune_fused_grid{-1};
std::atomic<int> g_tune_fused_max_rows{-1};
std::atomic<int> g_tune_prune{-1};
std::atomic<int> g_tune_select_wave{-1};
std::atomic<int> g_tune_part_rows{-1};
std::atomic<int> g_tune_remap{-1};
std::atomic<int> g_tune_nt{-1};
std::atomic<int> g_tune_vec{-1};
std::atomic<int> g_tune_poll{-1};
std::atomic<int> g_tune_coo_runs{-1};
std::atomic<int> g_tune_slab_shift{-1};

std::mutex g_mailbox_mutex;
FeatureRaw *g_mailbox_host = nullptr;   // pinned, mapped
FeatureRaw *g_mailbox_dev = nullptr;
uint64_t g_feature_seq = 0;

int hip_fail(hipError_t e)
{
    g_last_hip_error.store((int)e);
    return SEER_EHIP;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// x [cols] and y [rows] must be disjoint: every schedule reads x while other workgroups
// already write y.
bool vectors_overlap(const seer_csr *A, const float *x, const float *y)
{
    if (!x || !y) return false;
    const uintptr_t xb = reinterpret_cast<uintptr_t>(x), xe = xb + 4u * (uintptr_t)A->cols;
    const uintptr_t yb = reinterpret_cast<uintptr_t>(y), ye = yb + 4u * (uintptr_t)A->rows;
    return xb < ye && yb < xe;
}

int check_csr(const seer_csr *A, bool need_entries)
{
    if (!A) return SEER_EINVAL;
    if (A->rows < 0 || A->cols < 0 || A->nnz < 0) return SEER_EINVAL;
    if (!A->row_ptr) return SEER_EINVAL;
    if (need_entries && A->nnz > 0 && (!A->col_idx || !A->values)) return SEER_EINVAL;
    return SEER_OK;
}

int pow2_at_least(double v, int lo, int hi)
{
    int g = lo;
    while (g < hi && (double)g < v) g <<= 1;
    return g;
}

// Lanes per row for CSR,WM: the power of two at or above mean row length / 8, so that
// a lane walks about eight entries (two rounds of its four-way unrolled loop).
// Measured on banded and random matrices with mean lengths 5..200: wider groups
// lose up to 3x on banded rows, narrower ones at most ~15 % on random ones.  Small
// matrices get wider groups (below).
int wm_lanes(int rows, int nnz)
{
    const int t = g_tune_wm_lanes.load();
    if (t == 2 || t == 4 || t == 8 || t == 16 || t == 32 || t == 64) return t;
    const double mean = rows > 0 ? (double)nnz / (double)rows : 0.0;
    int g = pow2_at_least(mean / 8.0, 4, 64);   // (never two: four are 2 to 14 % faster on rows of 5 to 17, bands and random columns alike)
    // A matrix of up to half a million nonzeros is all latency: with every row's lanes
    // resident at once (the chip holds 2^19) a lane per entry, as far as the rows allow,
    // shortens each row's chain of dependent loads (4096 rows of 16: 4.2 -> 2.4 us, 16 000
    // rows of 16: 4.8 -> 3.5 us, 1000 rows of 100: 3.5 -> 2.6 us).  Larger matrices are
    // bound by the rate of the gathers and keep the narrow groups.
    if (rows > 0 && nnz <= (1 << 19)) {
        const int by_length = pow2_at_least(mean, 4, 64);
        int by_rows = 64;
        while (by_rows > 2 && (int64_t)rows * by_rows > ((int64_t)1 << 19)) by_rows /= 2;
        const int wide = by_length < by_rows ? by_length : by_rows;
        if (wide > g) g = wide;
    }
    return g;
}

// Rows per workgroup for CSR,BM, from measurements over banded / random matrices:
// short rows want fat blocks (5 K to 8 K nonzeros: fewer blocks, longer streams).  Rows
// longer than a wave get 16 per block, the most for which the kernel shares out the lanes
// among the rows (16 lanes each) -- fewer only where that would put more than 12 K
// nonzeros into a block (measured best at mean lengths 65 to 500: 16 rows; 1200: 4 to 8;
// 2000: 8).  A small matrix is cut finer (down to about one LDS chunk per block) so
// that every CU gets at least four blocks.
int bm_rows(int rows, int nnz)
{
    const int t = g_tune_bm_rows.load();
    if (t >= 1 && t <= kBmMaxRows) return t;
    const double mean = rows > 0 ? (double)nnz / (double)rows : 0.0;
    int r = 1;
    if (mean > 64.0) {
        r = 16;
        while (r > 1 && (double)r * mean > 12288.0) r >>= 1;
    } else {
        const double target = mean > 24.0 ? 8192.0 : 5120.0;
        while (r < 1024 && (double)r * mean * 1.41421356 < target) r <<= 1;   // nearest power of two
    }
    while (r > 1 && rows / r < 1024 && (double)r * mean > 2048.0) r >>= 1;
    return r;
}

// COO,WM sums an interval by lane-owned runs of triples unless the tuning knob asks for the
// rounds of 64.
bool coo_runs()
{
    return g_tune_coo_runs.load() != 0;
}

// Columns per slab of CSR,S, as a shift.  2^19 (2 MiB of x) keeps a slab inside an XCD's L2
// beside the streams; but where rows are short and the matrix is many slabs wide a row falls
// apart into pieces of one or two entries and the handling of the pieces costs more than the
// gathers save: with fewer than three entries per piece to expect (mean row length over the
// number of slabs) the slabs are 2^20 columns.  Measured on matrices of 2 M to 9 M rows: 0 to
// 20 % faster products below that mark (8 M rows of 23: 1917 -> 1600 us), 11 to 17 % slower
// above five entries per piece; 2^21 columns lose everywhere (x no longer stays in L2).
int slab_shift(int rows, int cols, int nnz)
{
    const int t = g_tune_slab_shift.load();
    if (t >= 1 && t <= 30) return t;
    const int64_t slabs = ((int64_t)cols + ((int64_t)1 << kSlabShift) - 1) >> kSlabShift;
    if (rows > 0 && slabs >= 4 && (int64_t)nnz < 3 * slabs * (int64_t)rows) return kSlabShift + 1;
    return kSlabShift;
}

int bm_chunk()
{
    const int t = g_tune_bm_chunk.load();
    return t == 4096 ? 4096 : kBmChunk;
}

int mp_ipt(int rows, int nnz)
{
    const int t = g_tune_mp_ipt.load();
    if (t == kMpIptSmall || t == kMpIptLarge) return t;
    // measured crossover: below ~6 M merge items the smaller tile (more workgroups) wins
    const uint64_t total = (uint64_t)rows + (uint64_t)nnz;
    return total < 6000000u ? kMpIptSmall : kMpIptLarge;
}

int auto_fused_rows()
{
    const int t = g_tune_fused_rows.load();
    return t < 0 ? kAutoFusedRows : t;
}

int use_remap()
{
    const int t = g_tune_remap.load();
    return t < 0 ? 1 : (t != 0);
}

// CSR,TM's own tile order.  With the XCD-contiguous order each XCD streams its own eighth of
// the arrays; from about 100 MB on, CSR,TM runs faster when consecutive tiles go to different
// XCDs and the whole chip moves through the arrays together (measured: 5-point stencils of
// 117 to 637 MB 2 to 4 % faster, the 872 MB one 10 %, bands of 3 to 7 per row 4 to 8 %,
// random columns unchanged; below about 75 MB the contiguous order wins by 3 to 5 %).  The
// other schedules gain or lose 2 to 4 % either way and keep the contiguous order.
int use_remap_tm(const seer_csr *A)
{
    const int t = g_tune_remap.load();
    if (t >= 0) return t != 0;
    const uint64_t bytes = 8ull * (uint64_t)A->nnz + 8ull * (uint64_t)A->rows + 4ull * (uint64_t)A->cols;
    return bytes <= (96ull << 20);
}

int use_nt()
{
    const int t = g_tune_nt.load();
    return t < 0 ? 1 : (t != 0);
}

// Products from a prepared plan are repeated with the same matrix.  If what a product reads
// and writes fits the caches (256 MB last-level cache + 8 x 4 MB L2), streaming it with the
// non-temporal hint gives up the reuse between products; beyond that size the hint keeps x
// in L2.  Measured, repeated products, plain against hinted loads: 212-218 MB (stencil, band,
// random columns) plain faster by 4 to 19 %; an 8 M-row 250 MB matrix 135 against 148-158 us;
// 325 MB stencil hinted faster by 10 % in the CSR kernels while ELL,TM, whose own arrays
// there come to 300 MB, is faster plain by 24 %; 424 MB and more hinted faster by 5 to 16 %.
// `footprint` is the byte count of the arrays the kernel reads and writes.
int use_nt_repeated(uint64_t footprint)
{
    const int t = g_tune_nt.load();
    if (t >= 0) return t != 0;
    return footprint > (288ull << 20);
}

uint64_t csr_footprint(const seer_csr *A)
{
    return 8ull * (uint64_t)A->nnz + 8ull * (uint64_t)A->rows + 4ull * (uint64_t)A->cols;
}

int ensure_mailbox()
{
    if (g_mailbox_host) return SEER_OK;
    void *h = nullptr;
    hipError_t e = hipHostMalloc(&h, 64, hipHostMallocPortable | hipHostMallocMapped);
    if (e != hipSuccess) return hip_fail(e);
    void *d = nullptr;
    e = hipHostGetDevicePointer(&d, h, 0);
    if (e != hipSuccess) {
        (void)hipHostFree(h);
        return hip_fail(e);
    }
    std::memset(h, 0, 64);
    g_mailbox_host = static_cast<FeatureRaw *>(h);
    g_mailbox_dev = static_cast<FeatureRaw *>(d);
    return SEER_OK;
}

// f[] from the exact integers; every entry is one fp64 quotient rounded once to fp32.
void derive(seer_features_t *o)
{
    for (int i = 0; i < SEER_NUM_FEATURES; ++i) o->f[i] = 0.0f;
    o->f[SEER_F_COLS] = (float)(double)o->cols;
    o->f[SEER_F_ITERATIONS] = 1.0f;
    if (o->rows <= 0) return;
    const double R = (double)o->rows;
    const double mean = (double)o->nnz / R;
    const unsigned __int128 num = (unsigned __int128)(uint64_t)o->rows * (unsigned __int128)o->sum_sq_len -
                                  (unsigned __int128)(uint64_t)o->nnz * (unsigned __int128)(uint64_t)o->nnz;
    const double var = (double)num / (double)((uint64_t)o->rows * (uint64_t)o->rows);
    o->f[SEER_F_ROWS] = (float)R;
    o->f[SEER_F_NNZ] = (float)(double)o->nnz;
    o->f[SEER_F_MEAN_LEN] = (float)mean;
    o->f[SEER_F_MAX_LEN] = (float)(double)o->max_len;
    o->f[SEER_F_MIN_LEN] = (float)(double)o->min_len;
    o->f[SEER_F_VAR_LEN] = (float)var;
    o->f[SEER_F_EMPTY_FRAC] = (float)((double)o->empty_rows / R);
    if (o->cols > 0) {
        const double C = (double)o->cols;
        o->f[SEER_F_MEAN_DENSITY] = (float)(mean / C);
        o->f[SEER_F_MAX_DENSITY] = (float)((double)o->max_len / C);
        o->f[SEER_F_MIN_DENSITY] = (float)((double)o->min_len / C);
        o->f[SEER_F_VAR_DENSITY] = (float)(var / (C * C));
    }
}

} // namespace

// Lays a validated, acyclic tree out as a complete binary tree of depth 6; false if some
// comparison lies deeper than that.
bool seer::flatten_tree(const seer_tree *t, AutoHeap *h)
{
    for (int i = 0; i < 64; ++i) { h->feature[i] = -1; h->threshold[i] = 0.0; }
    for (int i = 0; i < 128; ++i) h->klass[i] = (int8_t)SEER_CSR_MP;
    struct Item { int node, slot; };
    Item stack[256];
    int top = 0;
    stack[top++] = Item{0, 0};
    while (top > 0) {
        const Item it = stack[--top];
        const seer_node &nd = t->nodes[it.node];
        if (nd.feature < 0) {
            const int k = (nd.klass >= 0 && nd.klass < SEER_NUM_DIRECT_KERNELS) ? nd.klass : SEER_CSR_MP;
            h->klass[it.slot] = (int8_t)k;
            continue;                                  // feature[slot] stays -1 for slots below 63
        }
        if (it.slot >= kHeapInternal) return false;    // a comparison on the seventh level
        h->feature[it.slot] = nd.feature;
        h->threshold[it.slot] = nd.threshold;
        stack[top++] = Item{nd.left, 2 * it.slot + 1};
        stack[top++] = Item{nd.right, 2 * it.slot + 2};
    }
    return true;
}

namespace {

// every leaf names a kernel id below `limit`
bool leaves_below(const seer_tree *t, int limit)
{
    for (int i = 0; i < t->n_nodes; ++i)
        if (t->nodes[i].feature < 0 && t->nodes[i].klass >= limit) return false;
    return true;
}

// Classes of the leaves a walk can end in when only the entries of f[] that follow from
// rows, cols and nnz (and the iteration count) are known and the others may take any value:
// one bit per class.  The known comparisons are the ones seer_select and the device make,
// on the same bits.  Nodes may share children, so each is visited once; `seen` and `stack`
// hold n_nodes and 2 * n_nodes + 1 entries.  Classes must be below 32.
uint32_t reachable_classes(const seer_tree *t, const float *f, bool *seen, int32_t *stack)
{
    const auto known = [](int feature) {
        return feature == SEER_F_ROWS || feature == SEER_F_COLS || feature == SEER_F_NNZ ||
               feature == SEER_F_MEAN_LEN || feature == SEER_F_MEAN_DENSITY || feature == SEER_F_ITERATIONS;
    };
    uint32_t mask = 0;
    for (int32_t i = 0; i < t->n_nodes; ++i) seen[i] = false;
    int top = 0;
    stack[top++] = 0;
    while (top > 0) {
        const int32_t v = stack[--top];
        if (seen[v]) continue;
        seen[v] = true;
        const seer_node &nd = t->nodes[v];
        if (nd.feature < 0) {
            mask |= 1u << nd.klass;
        } else if (known(nd.feature)) {
            stack[top++] = ((double)f[nd.feature] <= nd.threshold) ? nd.left : nd.right;
        } else {
            stack[top++] = nd.left;
            stack[top++] = nd.right;
        }
    }
    return mask;
}

// ... for the asynchronous path, whose trees have at most kAutoMaxNodes nodes and only
// kernel ids below SEER_NUM_DIRECT_KERNELS in their leaves: nothing is allocated.
uint32_t reachable_kernels(const seer_tree *t, const float *f)
{
    bool seen[kAutoMaxNodes];
    int32_t stack[2 * kAutoMaxNodes + 1];
    return reachable_classes(t, f, seen, stack);
}

int check_tree(const seer_tree *t)
{
    if (!t->nodes || t->n_nodes < 1 || t->n_classes < 1 || t->n_features < 0 ||
        t->n_features > SEER_NUM_FEATURES)
        return SEER_ETREE;
    for (int32_t n = 0; n < t->n_nodes; ++n) {
        const seer_node &nd = t->nodes[n];
        if (nd.feature < 0) {
            if (nd.klass < 0 || nd.klass >= t->n_classes) return SEER_ETREE;
        } else {
            if (nd.feature >= t->n_features) return SEER_ETREE;
            if (nd.left < 0 || nd.left >= t->n_nodes || nd.right < 0 || nd.right >= t->n_nodes) return SEER_ETREE;
            if (nd.threshold != nd.threshold) return SEER_ETREE;   // NaN
        }
    }
    return SEER_OK;
}

// True if no path from the root visits a node twice (iterative depth-first walk).  Called
// with at most kAutoMaxNodes nodes, so its bookkeeping lives on the stack: the asynchronous
// entry points allocate nothing, on the host or the device.
bool tree_is_acyclic(const seer_tree *t)
{
    const int32_t n = t->n_nodes;
    if (n > kAutoMaxNodes) return false;
    uint8_t state[kAutoMaxNodes] = {};          // 0 unseen, 1 on the current path, 2 done
    int32_t stack[2 * kAutoMaxNodes + 1];       // a node is pushed at most once per parent edge
    int top = 0;
    stack[top++] = 0;
    while (top > 0) {
        const int32_t v = stack[top - 1];
        if (state[v] == 0) {
            state[v] = 1;
            const seer_node &nd = t->nodes[v];
            if (nd.feature >= 0) {
                for (int32_t c : {nd.left, nd.right}) {
                    if (state[c] == 1) return false;
                    if (state[c] == 0) {
                        if (top >= (int)(sizeof stack / sizeof stack[0])) return false;
                        stack[top++] = c;
                    }
                }
            }
        } else {
            if (state[v] == 1) state[v] = 2;
            --top;
        }
    }
    return true;
}

const char *const kKernelNames[SEER_NUM_KERNELS] = {"CSR,TM", "CSR,WM", "CSR,BM", "CSR,MP", "CSR,WO", "CSR,A", "ELL,TM", "COO,WM", "CSR,S"};

} // namespace

extern "C" {

int seer_num_kernels(void) { return SEER_NUM_KERNELS; }

const char *seer_kernel_name(int k) { return (k >= 0 && k < SEER_NUM_KERNELS) ? kKernelNames[k] : nullptr; }

const char *seer_strerror(int s)
{
    switch (s) {
    case SEER_OK: return "ok";
    case SEER_EINVAL: return "invalid argument";
    case SEER_EKERNEL: return "kernel id out of range";
    case SEER_ETREE: return "malformed decision tree";
    case SEER_EWORKSPACE: return "workspace missing, misaligned or too small";
    case SEER_EHIP: return "HIP runtime error";
    case SEER_ELIMIT: return "matrix too large for the library's built-in scratch";
    default: return "unknown status";
    }
}

int seer_last_hip_error(void) { return g_last_hip_error.load(); }

int seer_set_tuning(const char *name, int value)
{
    if (!name) return SEER_EINVAL;
    if (!std::strcmp(name, "wm_lanes")) g_tune_wm_lanes.store(value);
    else if (!std::strcmp(name, "bm_rows")) g_tune_bm_rows.store(value);
    else if (!std::strcmp(name, "bm_chunk")) g_tune_bm_chunk.store(value);
    else if (!std::strcmp(name, "mp_ipt")) g_tune_mp_ipt.store(value);
    else if (!std::strcmp(name, "auto_fused_rows")) g_tune_fused_rows.store(value);
    else if (!std::strcmp(name, "auto_fused_grid")) g_tune_fused_grid.store(value);
    else if (!std::strcmp(name, "auto_fused_max_rows")) g_tune_fused_max_rows.store(value);
    else if (!std::strcmp(name, "auto_prune")) g_tune_prune.store(value);
    else if (!std::strcmp(name, "auto_select_wave")) g_tune_select_wave.store(value);
    else if (!std::strcmp(name, "auto_part_rows")) g_tune_part_rows.store(value);
    else if (!std::strcmp(name, "xcd_remap")) g_tune_remap.store(value);
    else if (!std::strcmp(name, "nt")) g_tune_nt.store(value);
    else if (!std::strcmp(name, "vec")) g_tune_vec.store(value);
    else if (!std::strcmp(name, "poll")) g_tune_poll.store(value);
    else if (!std::strcmp(name, "coo_runs")) g_tune_coo_runs.store(value);
    else if (!std::strcmp(name, "slab_shift")) g_tune_slab_shift.store(value);
    else return SEER_EINVAL;
    return SEER_OK;
}

size_t seer_features_workspace_bytes(int32_t rows) { return rows < 0 ? 0 : features_workspace_bytes(rows); }

size_t seer_spmv_workspace_bytes(int kernel_id, int32_t rows, int32_t nnz)
{
    if (rows <= 0 || nnz < 0) return 0;
    if (kernel_id == SEER_CSR_WO) return carry_workspace_bytes(wo_num_tiles(rows, nnz));
    if (kernel_id == SEER_CSR_A)   // the carries, then the plan that the call builds for itself
        return carry_workspace_bytes(adaptive_num_tiles(rows, nnz)) + adaptive_plan_bytes(rows, nnz);
    if (kernel_id == SEER_COO_WM)
        return carry_workspace_bytes(coo_num_intervals(rows, nnz)) + coo_plan_bytes(rows, nnz);
    if (kernel_id != SEER_CSR_MP) return 0;
    // the small tile gives the larger count; cover either choice
    return mp_workspace_bytes(rows, nnz, kMpIptSmall);
}

int seer_derive_features(seer_features_t *io)
{
    if (!io) return SEER_EINVAL;
    if (io->rows < 0 || io->cols < 0 || io->nnz < 0 || io->max_len < 0 || io->min_len < 0 ||
        io->empty_rows < 0 || io->min_len > io->max_len || io->empty_rows > io->rows)
        return SEER_EINVAL;
    // rows * sum_sq >= nnz^2 holds for every real matrix (Cauchy-Schwarz); refuse anything else
    if ((unsigned __int128)(uint64_t)io->rows * io->sum_sq_len <
        (unsigned __int128)(uint64_t)io->nnz * (uint64_t)io->nnz)
        return SEER_EINVAL;
    derive(io);
    return SEER_OK;
}

int seer_known_features(int32_t rows, int32_t cols, int32_t nnz, seer_features_t *out)
{
    if (!out || rows < 0 || cols < 0 || nnz < 0) return SEER_EINVAL;
    seer_features_t o;
    std::memset(&o, 0, sizeof o);
    o.rows = rows; o.cols = cols; o.nnz = nnz;
    o.f[SEER_F_ROWS] = (float)(double)rows;
    o.f[SEER_F_COLS] = (float)(double)cols;
    o.f[SEER_F_NNZ] = (float)(double)nnz;
    o.f[SEER_F_ITERATIONS] = 1.0f;
    if (rows > 0) {
        const double mean = (double)nnz / (double)rows;
        o.f[SEER_F_MEAN_LEN] = (float)mean;
        if (cols > 0) o.f[SEER_F_MEAN_DENSITY] = (float)(mean / (double)cols);
    }
    *out = o;
    return SEER_OK;
}

int seer_features(const seer_csr *A, seer_features_t *out, void *workspace, size_t workspace_bytes,
                  void *stream)
{
    const int rc = check_csr(A, false);
    if (rc != SEER_OK) return rc;
    if (!out) return SEER_EINVAL;
    seer_features_t o;
    std::memset(&o, 0, sizeof o);
    o.rows = A->rows;
    o.cols = A->cols;
    if (A->rows > 0) {
        if (!workspace || !aligned16(workspace) || workspace_bytes < features_workspace_bytes(A->rows))
            return SEER_EWORKSPACE;
        std::lock_guard<std::mutex> lock(g_mailbox_mutex);
        const int mrc = ensure_mailbox();
        if (mrc != SEER_OK) return mrc;
        hipStream_t st = static_cast<hipStream_t>(stream);
        const uint64_t seq = ++g_feature_seq;
        launch_features(A->rows, A->row_ptr, workspace, g_mailbox_dev, seq, st);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
        // The kernel writes the statistics, then the sequence number, into pinned host
        // memory.  Watching that word is quicker than waiting for the stream; if it does
        // not show up soon, wait for the stream and look again.
        volatile uint64_t *seq_word = &g_mailbox_host->seq;
        bool seen = false;
        if (g_tune_poll.load() != 0) {
            const auto t0 = std::chrono::steady_clock::now();
            for (uint32_t spin = 0;; ++spin) {
                if (*seq_word == seq) { seen = true; break; }
                if ((spin & 1023u) == 1023u &&
                    std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(2))
                    break;
                __builtin_ia32_pause();
            }
        }
        if (!seen) {
            e = hipStreamSynchronize(st);
            if (e != hipSuccess) return hip_fail(e);
            if (*seq_word != seq) return hip_fail(hipErrorUnknown);
        }
        std::atomic_thread_fence(std::memory_order_acquire);
        FeatureRaw raw;
        std::memcpy(&raw, const_cast<const FeatureRaw *>(g_mailbox_host), sizeof raw);
        o.nnz = (int64_t)raw.last - (int64_t)raw.first;
        o.max_len = raw.max_len;
        o.min_len = raw.min_len;
        o.empty_rows = (int64_t)raw.empty;
        o.sum_sq_len = raw.sum_sq;
    }
    derive(&o);
    *out = o;
    return SEER_OK;
}

int seer_select(const seer_features_t *f, const seer_tree *t, int *kernel_id)
{
    if (!f || !t || !kernel_id) return SEER_EINVAL;
    const int rc = check_tree(t);
    if (rc != SEER_OK) return rc;
    int32_t n = 0;
    for (int32_t steps = 0; steps <= t->n_nodes; ++steps) {
        const seer_node &nd = t->nodes[n];
        if (nd.feature < 0) {
            *kernel_id = nd.klass;
            return SEER_OK;
        }
        n = ((double)f->f[nd.feature] <= nd.threshold) ? nd.left : nd.right;
    }
    return SEER_ETREE;   // walked more nodes than exist: a cycle
}

int seer_tree_reachable(const seer_tree *tree, const seer_features_t *known, uint32_t *class_mask)
{
    if (!tree || !known || !class_mask) return SEER_EINVAL;
    const int rc = check_tree(tree);
    if (rc != SEER_OK) return rc;
    if (tree->n_classes > 32) return SEER_ETREE;
    const size_t n = (size_t)tree->n_nodes;
    bool *seen = static_cast<bool *>(std::malloc(n));
    int32_t *stack = static_cast<int32_t *>(std::malloc((2 * n + 1) * sizeof(int32_t)));
    if (!seen || !stack) {
        std::free(seen);
        std::free(stack);
        return SEER_EINVAL;
    }
    *class_mask = reachable_classes(tree, known->f, seen, stack);
    std::free(seen);
    std::free(stack);
    return SEER_OK;
}

size_t seer_spmv_auto_workspace_bytes(int32_t rows, int32_t nnz)
{
    if (rows < 0 || nnz < 0) return 0;
    return auto_workspace_bytes(rows, nnz);
}

// Everything seer_spmv_auto checks before it needs scratch memory.  SEER_OK with *enqueue
// false: nothing to do (no rows).
static int auto_check(const seer_csr *A, const seer_tree *tree, const float *x, float *y, bool *enqueue)
{
    *enqueue = false;
    const int rc = check_csr(A, true);
    if (rc != SEER_OK) return rc;
    if (!tree) return SEER_EINVAL;
    const int trc = check_tree(tree);
    if (trc != SEER_OK) return trc;
    if (tree->n_nodes > kAutoMaxNodes || tree->n_classes > SEER_NUM_KERNELS) return SEER_ETREE;
    if (!leaves_below(tree, SEER_NUM_DIRECT_KERNELS)) return SEER_ETREE;
    // a cycle is only found by walking; make sure no walk can be longer than the tree
    if (!tree_is_acyclic(tree)) return SEER_ETREE;
    if (A->rows == 0) return SEER_OK;
    if (!y || (!x && A->nnz > 0) || vectors_overlap(A, x, y)) return SEER_EINVAL;
    *enqueue = true;
    return SEER_OK;
}

// Launch shapes from rows and nnz, then the launches; `workspace` holds at least
// auto_workspace_bytes(rows, nnz) bytes.
static int auto_enqueue(const seer_csr *A, const seer_tree *tree, const float *x, float *y, void *workspace,
                        void *stream)
{
    AutoTree dt;
    std::memset(&dt, 0, sizeof dt);
    dt.n_nodes = tree->n_nodes;
    std::memcpy(dt.nodes, tree->nodes, sizeof(seer_node) * (size_t)tree->n_nodes);
    AutoShape sh;
    sh.wm_lanes = wm_lanes(A->rows, A->nnz);
    sh.bm_rows = std::min(bm_rows(A->rows, A->nnz), kAutoBmMaxRows);   // (more only through the tuning knob)
    sh.bm_own_shift = bm_own_shift(sh.bm_rows);
    sh.mp_ipt = mp_ipt(A->rows, A->nnz);
    sh.tm_short = tm_short_rows(A->rows, A->nnz);
    sh.tm_pair = tm_rows_per_lane(A->rows, A->nnz) == 2;
    sh.tm_remap = use_remap_tm(A);
    const uint32_t rows = (uint32_t)A->rows;
    sh.tiles[SEER_CSR_TM] = tm_num_tiles(A->rows, A->nnz);
    sh.tiles[SEER_CSR_WM] = (rows + (256u / sh.wm_lanes) - 1u) / (256u / sh.wm_lanes);
    sh.tiles[SEER_CSR_BM] = (rows + (uint32_t)sh.bm_rows - 1u) / (uint32_t)sh.bm_rows;
    sh.tiles[SEER_CSR_MP] = mp_num_tiles(A->rows, A->nnz, sh.mp_ipt);
    sh.tiles[SEER_CSR_WO] = wo_num_tiles(A->rows, A->nnz);
    SpmvArgs a{A->rows, A->cols, A->nnz, A->row_ptr, A->col_idx, A->values, x, y, use_remap(), 1};
    const bool vec = aligned16(A->col_idx) && aligned16(A->values) && g_tune_vec.load() != 0;
    // What the host knows without looking at the matrix prunes the tree: the grid is sized
    // for the schedules that stay reachable, the carry fix-up is enqueued only if merge path
    // or the nonzero split is among them, and if a single kernel is left nothing is gathered.
    seer_features_t kf;
    (void)seer_known_features(A->rows, A->cols, A->nnz, &kf);
    sh.reachable = g_tune_prune.load() == 0 ? (1u << SEER_NUM_DIRECT_KERNELS) - 1u : reachable_kernels(tree, kf.f);
    AutoSel record;
    const bool decided = (sh.reachable & (sh.reachable - 1u)) == 0;
    if (decided) {
        std::memset(&record, 0, sizeof record);
        record.kernel_id = __builtin_ctz(sh.reachable);
        record.valid = 2;
        record.rows = A->rows; record.cols = A->cols; record.nnz = A->nnz;
        record.max_len = -1; record.min_len = -1;
        record.empty = ~0ull;
        for (int i = 0; i < SEER_NUM_FEATURES; ++i) record.f[i] = kf.f[i];
    }
    const int fg = g_tune_fused_grid.load(), fm = g_tune_fused_max_rows.load();
    const int pr = g_tune_part_rows.load();
    const AutoPolicy policy{auto_fused_rows(), fg < 0 ? kAutoFusedGrid : fg, fm < 0 ? kAutoFusedMaxRows : fm,
                            g_tune_select_wave.load() != 0, pr >= 256 ? (uint32_t)pr : 0u};
    AutoHeap heap;
    const bool flat = flatten_tree(tree, &heap);
    launch_auto(a, dt, flat ? &heap : nullptr, sh, vec, policy, decided ? &record : nullptr, workspace,
                static_cast<hipStream_t>(stream));
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? SEER_OK : hip_fail(e);
}

int seer_spmv_auto(const seer_csr *A, const seer_tree *tree, const float *x, float *y, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    bool enqueue = false;
    const int rc = auto_check(A, tree, x, y, &enqueue);
    if (rc != SEER_OK || !enqueue) return rc;
    if (!workspace || !aligned16(workspace) || workspace_bytes < auto_workspace_bytes(A->rows, A->nnz))
        return SEER_EWORKSPACE;
    return auto_enqueue(A, tree, x, y, workspace, stream);
}

int seer_spmv_auto_static(const seer_csr *A, const seer_tree *tree, const float *x, float *y, void *stream)
{
    bool enqueue = false;
    const int rc = auto_check(A, tree, x, y, &enqueue);
    if (rc != SEER_OK || !enqueue) return rc;
    if (auto_workspace_bytes(A->rows, A->nnz) > kStaticScratchBytes) return SEER_ELIMIT;
    // The array's device address, looked up once per device with that device current.
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return SEER_EINVAL;
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return hip_fail(e);
            if (!p) return hip_fail(hipErrorInvalidSymbol);
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    return auto_enqueue(A, tree, x, y, ptr, stream);
}

int seer_spmv_model(const seer_csr *A, const seer_model *model, const float *x, float *y, void *workspace,
                    size_t workspace_bytes, void *stream, int *path, int *kernel_id)
{
    if (!A) return SEER_EINVAL;
    if (model && (!model->gathered || (model->selector && !model->known))) return SEER_EINVAL;
    if (A->rows < 0 || A->cols < 0 || A->nnz < 0) return SEER_EINVAL;
    int use_gathered = 1;
    int kid = -1;
    const seer_tree *gathered = model ? model->gathered : &seer_model_gathered_tree;
    if (!model) {                       // the built-in models: generated code for the two host-side trees
        seer_features_t kf;
        const int rc = seer_known_features(A->rows, A->cols, A->nnz, &kf);
        if (rc != SEER_OK) return rc;
        use_gathered = seer_model_selector(kf.f) != 0;
        if (!use_gathered) kid = seer_model_known(kf.f);
    } else if (model->selector) {
        seer_features_t kf;
        int rc = seer_known_features(A->rows, A->cols, A->nnz, &kf);
        if (rc != SEER_OK) return rc;
        if (model->selector->n_classes > 2) return SEER_ETREE;
        rc = seer_select(&kf, model->selector, &use_gathered);
        if (rc != SEER_OK) return rc;
        if (!use_gathered) {
            if (model->known->n_classes > SEER_NUM_KERNELS) return SEER_ETREE;
            rc = seer_select(&kf, model->known, &kid);
            if (rc != SEER_OK) return rc;
        }
    }
    if (!use_gathered && (kid < 0 || kid >= SEER_NUM_DIRECT_KERNELS)) return SEER_ETREE;   // needs preprocessing: seer_spmv_plan
    if (A->rows > 0 && (!workspace || !aligned16(workspace) ||
                        workspace_bytes < auto_workspace_bytes(A->rows, A->nnz)))
        return SEER_EWORKSPACE;
    const int rc = use_gathered ? seer_spmv_auto(A, gathered, x, y, workspace, workspace_bytes, stream)
                                : seer_spmv(kid, A, x, y, workspace, workspace_bytes, stream);
    if (rc != SEER_OK) return rc;
    if (path) *path = use_gathered;
    if (kernel_id) *kernel_id = kid;
    return SEER_OK;
}

int seer_model_host_ns(const seer_model *model, int32_t rows, int32_t cols, int32_t nnz, int32_t reps, double *ns)
{
    if (!model || !model->selector || !model->known || !ns || reps < 1) return SEER_EINVAL;
    volatile int sink = 0;
    const auto t0 = std::chrono::steady_clock::now();
    for (int32_t i = 0; i < reps; ++i) {
        seer_features_t kf;
        int use_gathered = 1, kid = -1;
        int rc = seer_known_features(rows, cols, nnz, &kf);
        if (rc == SEER_OK) rc = seer_select(&kf, model->selector, &use_gathered);
        if (rc == SEER_OK && !use_gathered) rc = seer_select(&kf, model->known, &kid);
        if (rc != SEER_OK) return rc;
        sink = sink + use_gathered + kid;
    }
    const auto t1 = std::chrono::steady_clock::now();
    *ns = std::chrono::duration<double, std::nano>(t1 - t0).count() / (double)reps;
    return SEER_OK;
}

int seer_spmv_auto_result(const void *workspace, void *stream, seer_features_t *features, int *kernel_id)
{
    if (!workspace) return SEER_EINVAL;
    AutoSel sel;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(&sel, static_cast<const char *>(workspace) + kAutoSelOffset, sizeof sel,
                                  hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e);
    if (sel.valid != 1 && sel.valid != 2) return SEER_EINVAL;
    if (kernel_id) *kernel_id = sel.kernel_id;
    if (features) {
        std::memset(features, 0, sizeof *features);
        features->nnz = sel.nnz;
        features->max_len = sel.max_len;
        features->min_len = sel.min_len;
        features->empty_rows = (int64_t)sel.empty;
        features->sum_sq_len = sel.sum_sq;
        features->rows = sel.rows;
        features->cols = sel.cols;
        for (int i = 0; i < SEER_NUM_FEATURES; ++i) features->f[i] = sel.f[i];
    }
    return SEER_OK;
}

int seer_stream_copy(void *dst, const void *src, size_t n_words, void *stream)
{
    if (n_words == 0) return SEER_OK;
    if (!dst || !src || !aligned16(dst) || !aligned16(src)) return SEER_EINVAL;
    launch_stream_copy(dst, src, n_words, static_cast<hipStream_t>(stream));
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? SEER_OK : hip_fail(e);
}

int seer_csr_check(const seer_csr *A, int64_t *bad_row_ptr, int64_t *bad_col_idx, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    if (!A || !bad_row_ptr || !bad_col_idx) return SEER_EINVAL;
    if (A->rows < 0 || A->cols < 0 || A->nnz < 0 || !A->row_ptr) return SEER_EINVAL;
    if (!workspace || !aligned16(workspace) || workspace_bytes < 16) return SEER_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemsetAsync(workspace, 0, 16, st);
    if (e != hipSuccess) return hip_fail(e);
    launch_csr_check(A->rows, A->cols, A->nnz, A->row_ptr, A->col_idx, workspace, st);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    unsigned long long counts[2] = {0, 0};
    e = hipMemcpyAsync(counts, workspace, sizeof counts, hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e);
    *bad_row_ptr = (int64_t)counts[0];
    *bad_col_idx = (int64_t)counts[1];
    return SEER_OK;
}

int seer_stream_sum(const void *src, size_t n_words, void *out64, void *stream)
{
    if (n_words == 0) return SEER_OK;
    if (!src || !out64 || !aligned16(src)) return SEER_EINVAL;
    launch_stream_sum(src, n_words, out64, static_cast<hipStream_t>(stream));
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? SEER_OK : hip_fail(e);
}

int seer_gather_sum(const int32_t *idx, const float *val, size_t n, const float *x, void *out64, void *stream)
{
    if (n < 4) return SEER_OK;
    if (!idx || !val || !x || !out64 || !aligned16(idx) || !aligned16(val)) return SEER_EINVAL;
    launch_gather_sum(idx, val, n, x, out64, static_cast<hipStream_t>(stream));
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? SEER_OK : hip_fail(e);
}

static int spmv_dispatch(int kernel_id, const seer_csr *A, const float *x, float *y, void *workspace,
                         size_t workspace_bytes, void *stream, int nt);

int seer_spmv(int kernel_id, const seer_csr *A, const float *x, float *y, void *workspace,
              size_t workspace_bytes, void *stream)
{
    return spmv_dispatch(kernel_id, A, x, y, workspace, workspace_bytes, stream, use_nt());
}

static int spmv_dispatch(int kernel_id, const seer_csr *A, const float *x, float *y, void *workspace,
                         size_t workspace_bytes, void *stream, int nt)
{
    if (kernel_id < 0 || kernel_id >= SEER_NUM_KERNELS || kernel_id == SEER_ELL_TM || kernel_id == SEER_CSR_S)
        return SEER_EKERNEL;
    const int rc = check_csr(A, true);
    if (rc != SEER_OK) return rc;
    if (A->rows == 0) return SEER_OK;
    if (!y || (!x && A->nnz > 0) || vectors_overlap(A, x, y)) return SEER_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    SpmvArgs a{A->rows, A->cols, A->nnz, A->row_ptr, A->col_idx, A->values, x, y, use_remap(), nt};
    const bool vec = aligned16(A->col_idx) && aligned16(A->values) && g_tune_vec.load() != 0;
    switch (kernel_id) {
    case SEER_CSR_TM: {
        SpmvArgs t = a;
        t.remap = use_remap_tm(A);
        launch_tm(t, st);
        break;
    }
    case SEER_CSR_WM: launch_wm(a, wm_lanes(A->rows, A->nnz), st); break;
    case SEER_CSR_BM: launch_bm(a, bm_rows(A->rows, A->nnz), bm_chunk(), vec, st); break;
    case SEER_CSR_A: {
        // single call: the preprocessing pass runs first, on the same stream, every time
        const size_t carry = carry_workspace_bytes(adaptive_num_tiles(A->rows, A->nnz));
        if (!workspace || !aligned16(workspace) || workspace_bytes < carry + adaptive_plan_bytes(A->rows, A->nnz))
            return SEER_EWORKSPACE;
        void *plan_mem = static_cast<char *>(workspace) + carry;
        launch_adaptive_plan(A->rows, A->nnz, A->row_ptr, plan_mem, false, st);
        launch_adaptive(a, vec, plan_mem, workspace, st);
        break;
    }
    case SEER_COO_WM: {
        const size_t carry = carry_workspace_bytes(coo_num_intervals(A->rows, A->nnz));
        if (!workspace || !aligned16(workspace) || workspace_bytes < carry + coo_plan_bytes(A->rows, A->nnz))
            return SEER_EWORKSPACE;
        void *plan_mem = static_cast<char *>(workspace) + carry;
        launch_coo_convert(A->rows, A->row_ptr, plan_mem, st);
        launch_coo(a, coo_runs(), plan_mem, workspace, st);
        break;
    }
    case SEER_CSR_WO:
        if (!workspace || !aligned16(workspace) ||
            workspace_bytes < carry_workspace_bytes(wo_num_tiles(A->rows, A->nnz)))
            return SEER_EWORKSPACE;
        launch_wo(a, vec, workspace, st);
        break;
    default: {
        const int ipt = mp_ipt(A->rows, A->nnz);
        if (!workspace || !aligned16(workspace) || workspace_bytes < mp_workspace_bytes(A->rows, A->nnz, ipt))
            return SEER_EWORKSPACE;
        launch_mp(a, ipt, vec, workspace, st);
        break;
    }
    }
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? SEER_OK : hip_fail(e);
}

size_t seer_plan_bytes(int kernel_id, int32_t rows, int32_t nnz)
{
    if (rows <= 0 || nnz < 0) return 0;
    if (kernel_id == SEER_COO_WM) return coo_plan_bytes(rows, nnz);
    if (kernel_id != SEER_CSR_A) return 0;
    return adaptive_plan_bytes(rows, nnz);
}

size_t seer_ell_plan_bytes(int32_t rows, int32_t max_len) { return ell_plan_bytes(rows, max_len); }

size_t seer_slab_plan_bytes(int32_t rows, int32_t cols, int32_t nnz)
{
    if (rows < 0 || cols < 0 || nnz < 0) return 0;
    return slab_plan_bytes(rows, cols, nnz, slab_shift(rows, cols, nnz));
}

// The column-slabbed form: counts, the check of the column order and the number of virtual
// rows that hold entries; then, if every row's columns ascend, the offsets, the lists of
// pieces and the entries.
static int prepare_slab(const seer_csr *A, void *plan_mem, size_t plan_bytes, void *stream, seer_plan *plan)
{
    const int shift = slab_shift(A->rows, A->cols, A->nnz);
    const uint32_t S = slab_count(A->rows, A->cols, shift);
    if (S == 0) return SEER_EINVAL;                        // one slab, or too many virtual rows
    const size_t need = slab_plan_bytes(A->rows, A->cols, A->nnz, shift);
    plan->device_bytes = need;
    if (!plan_mem || !aligned16(plan_mem) || plan_bytes < need) return SEER_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    launch_slab_count(A->rows, A->cols, A->nnz, shift, A->row_ptr, A->col_idx, plan_mem, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    int descends = 0;
    uint32_t n_kept = 0;
    e = hipMemcpyAsync(&descends, slab_flag(plan_mem, A->rows, A->cols, A->nnz, shift), sizeof(int), hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return hip_fail(e);
    e = hipMemcpyAsync(&n_kept, slab_kept_count(plan_mem, A->rows, A->cols, A->nnz, shift), sizeof n_kept,
                       hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e);
    if (descends) return SEER_EINVAL;                      // a virtual row would not be one piece of its row
    if ((size_t)n_kept > (size_t)A->nnz) return hip_fail(hipErrorUnknown);
    launch_slab_fill(A->rows, A->cols, A->nnz, shift, n_kept, A->row_ptr, A->col_idx, A->values, plan_mem, st);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e);
    plan->n_blocks = (int32_t)S;
    plan->ell_width = shift;                               // kept with the plan: the knob may move afterwards
    plan->split_rows = (int32_t)n_kept;
    plan->device = plan_mem;
    return SEER_OK;
}

// The ELL conversion.  max_len < 0: not known yet, find it with the feature reduction.
static int prepare_ell(const seer_csr *A, void *plan_mem, size_t plan_bytes, void *stream, seer_plan *plan,
                       int64_t max_len)
{
    if (!plan_mem || !aligned16(plan_mem)) return SEER_EWORKSPACE;
    if (max_len < 0) {
        // the longest row is found with plan_mem as the reduction's workspace: it must hold that first
        if (plan_bytes < features_workspace_bytes(A->rows)) {
            plan->device_bytes = features_workspace_bytes(A->rows);
            return SEER_EWORKSPACE;
        }
        seer_features_t f;
        const int rc = seer_features(A, &f, plan_mem, plan_bytes, stream);
        if (rc != SEER_OK) return rc;
        max_len = f.max_len;
    }
    const size_t need = ell_plan_bytes(A->rows, (int)max_len);
    if (need == 0) return SEER_EINVAL;                 // 2^31 words or more: not applicable
    plan->device_bytes = need;
    if (plan_bytes < need) return SEER_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    launch_ell_convert(A->rows, (int)max_len, A->row_ptr, A->col_idx, A->values, plan_mem, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e);
    plan->ell_width = (int32_t)max_len;
    plan->device = plan_mem;
    return SEER_OK;
}

// seer_spmv_prepare into a plan of the library's own; the caller's is written on success only.
static int prepare_into(int kernel_id, const seer_csr *A, void *plan_mem, size_t plan_bytes, void *stream,
                        seer_plan *plan)
{
    std::memset(plan, 0, sizeof *plan);
    plan->kernel_id = kernel_id;
    plan->rows = A->rows;
    plan->nnz = A->nnz;
    if (kernel_id == SEER_ELL_TM && A->rows > 0) return prepare_ell(A, plan_mem, plan_bytes, stream, plan, -1);
    if (kernel_id == SEER_CSR_S) return A->rows > 0 ? prepare_slab(A, plan_mem, plan_bytes, stream, plan) : SEER_EINVAL;
    if (kernel_id == SEER_COO_WM && A->rows > 0) {
        const size_t need = coo_plan_bytes(A->rows, A->nnz);
        if (!plan_mem || !aligned16(plan_mem) || plan_bytes < need) return SEER_EWORKSPACE;
        hipStream_t st = static_cast<hipStream_t>(stream);
        launch_coo_convert(A->rows, A->row_ptr, plan_mem, st);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
        e = hipStreamSynchronize(st);
        if (e != hipSuccess) return hip_fail(e);
        plan->device = plan_mem;
        plan->device_bytes = need;
        return SEER_OK;
    }
    if (kernel_id != SEER_CSR_A || A->rows == 0) return SEER_OK;   // nothing to prepare
    const size_t need = adaptive_plan_bytes(A->rows, A->nnz);
    if (!plan_mem || !aligned16(plan_mem) || plan_bytes < need) return SEER_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int *flag = adaptive_split_flag(plan_mem, A->rows, A->nnz);
    hipError_t e = hipMemsetAsync(flag, 0, sizeof(int), st);
    if (e != hipSuccess) return hip_fail(e);
    launch_adaptive_plan(A->rows, A->nnz, A->row_ptr, plan_mem, true, st);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    int split = 0;
    e = hipMemcpyAsync(&split, flag, sizeof(int), hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e);
    plan->n_blocks = (int32_t)adaptive_num_tiles(A->rows, A->nnz);
    plan->split_rows = split != 0;
    plan->device = plan_mem;
    plan->device_bytes = need;
    return SEER_OK;
}

int seer_spmv_prepare(int kernel_id, const seer_csr *A, void *plan_mem, size_t plan_bytes, void *stream,
                      seer_plan *plan)
{
    if (!plan) return SEER_EINVAL;
    if (kernel_id < 0 || kernel_id >= SEER_NUM_KERNELS) return SEER_EKERNEL;
    const int rc = check_csr(A, true);
    if (rc != SEER_OK) return rc;
    seer_plan made;
    const int prc = prepare_into(kernel_id, A, plan_mem, plan_bytes, stream, &made);
    if (prc == SEER_OK) *plan = made;
    else if (prc == SEER_EWORKSPACE && (kernel_id == SEER_ELL_TM || kernel_id == SEER_CSR_S))
        plan->device_bytes = made.device_bytes;            // the documented exception
    return prc;
}

size_t seer_spmv_prepared_workspace_bytes(const seer_plan *plan)
{
    if (!plan) return 0;
    if (plan->kernel_id == SEER_CSR_A)
        return plan->split_rows ? carry_workspace_bytes((uint32_t)plan->n_blocks) : 0;
    if (plan->kernel_id == SEER_ELL_TM) return 0;
    if (plan->kernel_id == SEER_CSR_S)      // one partial per kept virtual row, then CSR,WO's carries over them
        return plan->split_rows < 0 ? 0 : slab_workspace_bytes((uint32_t)plan->split_rows, plan->nnz);
    return seer_spmv_workspace_bytes(plan->kernel_id, plan->rows, plan->nnz);
}

int seer_spmv_prepared(const seer_plan *plan, const seer_csr *A, const float *x, float *y, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    if (!plan) return SEER_EINVAL;
    if (plan->kernel_id != SEER_CSR_A && plan->kernel_id != SEER_ELL_TM && plan->kernel_id != SEER_COO_WM &&
        plan->kernel_id != SEER_CSR_S)
        return spmv_dispatch(plan->kernel_id, A, x, y, workspace, workspace_bytes, stream,
                             A ? use_nt_repeated(csr_footprint(A)) : use_nt());
    const int rc = check_csr(A, true);
    if (rc != SEER_OK) return rc;
    if (A->rows != plan->rows || A->nnz != plan->nnz) return SEER_EINVAL;   // a plan belongs to one matrix
    if (A->rows == 0) return SEER_OK;
    if (!y || (!x && A->nnz > 0) || !plan->device || vectors_overlap(A, x, y)) return SEER_EINVAL;
    if (plan->kernel_id == SEER_COO_WM) {
        if (!workspace || !aligned16(workspace) ||
            workspace_bytes < carry_workspace_bytes(coo_num_intervals(A->rows, A->nnz)))
            return SEER_EWORKSPACE;
        SpmvArgs a{A->rows, A->cols, A->nnz, A->row_ptr, A->col_idx, A->values, x, y, use_remap(),
                   use_nt_repeated(csr_footprint(A) + 4ull * (uint64_t)A->nnz)};
        launch_coo(a, coo_runs(), plan->device, workspace, static_cast<hipStream_t>(stream));
        const hipError_t e = hipGetLastError();
        return e == hipSuccess ? SEER_OK : hip_fail(e);
    }
    if (plan->kernel_id == SEER_CSR_S) {
        if (plan->n_blocks < 2 || plan->split_rows < 0 || plan->split_rows > A->nnz) return SEER_EINVAL;
        if (!workspace || !aligned16(workspace) || workspace_bytes < seer_spmv_prepared_workspace_bytes(plan))
            return SEER_EWORKSPACE;
        SpmvArgs a{A->rows, A->cols, A->nnz, A->row_ptr, A->col_idx, A->values, x, y, use_remap(),
                   use_nt_repeated(8ull * (uint64_t)A->nnz + 4ull * ((uint64_t)A->cols + 2ull * (uint64_t)A->rows) +
                                   16ull * (uint64_t)plan->split_rows)};
        launch_slab(a, (uint32_t)plan->n_blocks, (uint32_t)plan->split_rows, plan->device, workspace,
                    static_cast<hipStream_t>(stream));
        const hipError_t e = hipGetLastError();
        return e == hipSuccess ? SEER_OK : hip_fail(e);
    }
    if (plan->kernel_id == SEER_ELL_TM) {
        SpmvArgs a{A->rows, A->cols, A->nnz, A->row_ptr, A->col_idx, A->values, x, y, use_remap(),
                   use_nt_repeated((uint64_t)plan->device_bytes + 4ull * ((uint64_t)A->rows + (uint64_t)A->cols))};
        launch_ell(a, plan->ell_width, plan->device, static_cast<hipStream_t>(stream));
        const hipError_t e = hipGetLastError();
        return e == hipSuccess ? SEER_OK : hip_fail(e);
    }
    void *carry = nullptr;
    if (plan->split_rows) {
        if (!workspace || !aligned16(workspace) ||
            workspace_bytes < carry_workspace_bytes((uint32_t)plan->n_blocks))
            return SEER_EWORKSPACE;
        carry = workspace;
    }
    SpmvArgs a{A->rows, A->cols, A->nnz, A->row_ptr, A->col_idx, A->values, x, y, use_remap(),
               use_nt_repeated(csr_footprint(A))};
    const bool vec = aligned16(A->col_idx) && aligned16(A->values) && g_tune_vec.load() != 0;
    launch_adaptive(a, vec, plan->device, carry, static_cast<hipStream_t>(stream));
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? SEER_OK : hip_fail(e);
}

int seer_spmv_plan(const seer_csr *A, const seer_model *model, int32_t iterations, void *plan_mem,
                   size_t plan_bytes, void *workspace, size_t workspace_bytes, void *stream, seer_plan *plan,
                   int *path)
{
    if (!A || !plan || iterations < 1) return SEER_EINVAL;
    if (model && (!model->gathered || (model->selector && !model->known))) return SEER_EINVAL;
    int rc = check_csr(A, true);
    if (rc != SEER_OK) return rc;
    int use_gathered = 1, kid = -1;
    int64_t max_len = -1;
    if (!model || model->selector) {
        seer_features_t kf;
        rc = seer_known_features(A->rows, A->cols, A->nnz, &kf);
        if (rc != SEER_OK) return rc;
        kf.f[SEER_F_ITERATIONS] = (float)iterations;
        if (!model) {                   // the built-in models for several products
            use_gathered = seer_model_iterative_selector(kf.f) != 0;
            if (!use_gathered) kid = seer_model_iterative_known(kf.f);
        } else {
            if (model->selector->n_classes > 2) return SEER_ETREE;
            rc = seer_select(&kf, model->selector, &use_gathered);
            if (rc != SEER_OK) return rc;
            if (!use_gathered) {
                rc = seer_select(&kf, model->known, &kid);
                if (rc != SEER_OK) return rc;
            }
        }
    }
    if (use_gathered) {
        seer_features_t gf;
        rc = seer_features(A, &gf, workspace, workspace_bytes, stream);
        if (rc != SEER_OK) return rc;
        gf.f[SEER_F_ITERATIONS] = (float)iterations;
        max_len = gf.max_len;
        if (!model) {
            kid = seer_model_iterative_gathered(gf.f);
        } else {
            rc = seer_select(&gf, model->gathered, &kid);
            if (rc != SEER_OK) return rc;
        }
    }
    if (kid < 0 || kid >= SEER_NUM_KERNELS) return SEER_ETREE;
    seer_plan made;
    if (kid == SEER_ELL_TM && A->rows > 0) {
        std::memset(&made, 0, sizeof made);
        made.kernel_id = kid;
        made.rows = A->rows;
        made.nnz = A->nnz;
        rc = prepare_ell(A, plan_mem, plan_bytes, stream, &made, max_len);
        if (rc == SEER_OK) {
            *plan = made;
            if (path) *path = use_gathered;
            return SEER_OK;
        }
        if (rc != SEER_EWORKSPACE && rc != SEER_EINVAL) return rc;
        kid = SEER_CSR_A;            // the ELL arrays do not fit: take the schedule that is safe everywhere
    }
    if (kid == SEER_CSR_S) {
        rc = prepare_into(kid, A, plan_mem, plan_bytes, stream, &made);
        if (rc == SEER_OK) {
            *plan = made;
            if (path) *path = use_gathered;
            return SEER_OK;
        }
        if (rc != SEER_EWORKSPACE && rc != SEER_EINVAL) return rc;
        kid = SEER_CSR_A;            // no room for the second copy, or the form does not apply
    }
    rc = prepare_into(kid, A, plan_mem, plan_bytes, stream, &made);
    if (rc != SEER_OK) return rc;
    *plan = made;                    // outputs are written on success only
    if (path) *path = use_gathered;
    return SEER_OK;
}

} // extern "C"
