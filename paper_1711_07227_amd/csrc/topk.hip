// Top-k per query (Sec. III: the k smallest distances of a row of the result and the positions of the
// respective database histograms, stored in the n2 x k matrix R).  D is n x q row-major here, so a query
// is a column; lanes run along 32 neighbouring columns to keep the reads of D contiguous, and the rows
// are split over workgroups.  Order everywhere: (distance, row index) ascending.
#include <float.h>
#include <limits.h>

#include "lcrwmd_internal.h"

namespace lcrwmd {

namespace {

constexpr int COLS = 32;     // query columns per workgroup
constexpr int LISTS = 8;     // row lanes per column (256 threads = 32 x 8)

struct TopkPlan {
    int64_t col_strips;
    int32_t nsplit;
    int64_t rows_per_split;
};

TopkPlan plan_topk(int64_t n, int64_t q, int k, size_t ws_bytes)
{
    TopkPlan p;
    p.col_strips = (q + COLS - 1) / COLS;
    int64_t want = (2048 + p.col_strips - 1) / p.col_strips;    // aim at ~2k workgroups
    int64_t by_rows = n / 2048 > 0 ? n / 2048 : 1;                 // at least ~2k rows per split
    int64_t ns = want < by_rows ? want : by_rows;
    if (ns > 64) ns = 64;
    if (ns < 1) ns = 1;
    size_t need = (size_t)ns * (size_t)q * (size_t)k * 8;
    if (ns > 1 && need > ws_bytes) ns = 1;
    p.nsplit = (int32_t)ns;
    p.rows_per_split = (n + ns - 1) / ns;
    return p;
}

__device__ inline bool before(float d, int32_t i, float bd, int32_t bi) { return d < bd || (d == bd && i < bi); }

// Partial top-k of rows [split * rows_per_split, ...) for 32 columns.
// bound (or null): bound[j * k + k - 1] is a distance that k rows seen EARLIER (smaller row indices) already reach for
// column j - the running list of lcrwmd_rwmd_reduce.  Only strictly smaller values can still enter the final list (an
// equal one loses the tie on its row index), so everything else is skipped without touching the lists: after the
// first blocks of a long database almost every value is.
__global__ __launch_bounds__(256) void k_topk_partial(const float* __restrict__ D, int64_t n, int64_t q,
                                                      int64_t ldd, int k, int64_t rows_per_split,
                                                      int64_t col_strips, const float* __restrict__ bound,
                                                      float* __restrict__ out_d, int32_t* __restrict__ out_i)
{
    extern __shared__ unsigned char smem[];
    float* kd = reinterpret_cast<float*>(smem);                          // [k][256]
    int32_t* ki = reinterpret_cast<int32_t*>(smem + (size_t)k * 256 * 4);  // [k][256]
    int32_t* cnt_s = reinterpret_cast<int32_t*>(smem + (size_t)k * 256 * 8);

    const int tid = threadIdx.x;
    const int jj = tid & (COLS - 1), rg = tid / COLS;
    const int64_t strip = blockIdx.x % col_strips;
    const int64_t split = blockIdx.x / col_strips;
    const int64_t j = strip * COLS + jj;
    const int64_t r_begin = split * rows_per_split;
    int64_t r_end = r_begin + rows_per_split;
    if (r_end > n) r_end = n;

    int cnt = 0;
    const float outer = (bound && j < q) ? bound[j * k + k - 1] : FLT_MAX;
    float worst = outer;               // values not below this cannot enter the list
    auto offer = [&](float d, int64_t i) {
        if (!(d < worst)) return;
        int pos = cnt < k ? cnt++ : k - 1;
        while (pos > 0 && d < kd[(pos - 1) * 256 + tid]) {
            kd[pos * 256 + tid] = kd[(pos - 1) * 256 + tid];
            ki[pos * 256 + tid] = ki[(pos - 1) * 256 + tid];
            --pos;
        }
        kd[pos * 256 + tid] = d;
        ki[pos * 256 + tid] = (int32_t)i;
        if (cnt == k) worst = fminf(outer, kd[(k - 1) * 256 + tid]);
    };
    if (j < q) {
        // eight rows' values are requested before the first is looked at: a list rarely changes once it is full, so
        // the loop is a stream of loads whose latency must overlap
        constexpr int UN = 8;
        int64_t i = r_begin + rg;
        for (; i + (UN - 1) * LISTS < r_end; i += UN * LISTS) {
            float d[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) d[u] = D[(i + u * LISTS) * ldd + j];
#pragma unroll
            for (int u = 0; u < UN; ++u) offer(d[u], i + u * LISTS);
        }
        for (; i < r_end; i += LISTS) offer(D[i * ldd + j], i);
    }
    cnt_s[tid] = cnt;
    __syncthreads();
    if (rg == 0 && j < q) {
        int h[LISTS];
#pragma unroll
        for (int g = 0; g < LISTS; ++g) h[g] = 0;
        float* od = out_d + ((size_t)split * q + j) * k;
        int32_t* oi = out_i + ((size_t)split * q + j) * k;
        for (int r = 0; r < k; ++r) {
            int best = -1;
            float bd = FLT_MAX;
            int32_t bi = INT_MAX;
#pragma unroll
            for (int g = 0; g < LISTS; ++g) {
                const int t = jj + COLS * g;
                if (h[g] < cnt_s[t]) {
                    const float d = kd[h[g] * 256 + t];
                    const int32_t i = ki[h[g] * 256 + t];
                    if (best < 0 || before(d, i, bd, bi)) { best = g; bd = d; bi = i; }
                }
            }
            od[r] = bd;      // FLT_MAX / INT_MAX mark a slot this split could not fill
            oi[r] = bi;
#pragma unroll
            for (int g = 0; g < LISTS; ++g)
                if (best == g) ++h[g];
        }
    }
}

// One wavefront per query merges the nsplit (<= 64) sorted partial lists.
__global__ __launch_bounds__(64) void k_topk_merge(const float* __restrict__ part_d, const int32_t* __restrict__ part_i,
                                                   int64_t q, int k, int nsplit, float* __restrict__ R_dist,
                                                   int32_t* __restrict__ R_idx)
{
    const int64_t j = blockIdx.x;
    const int lane = threadIdx.x;
    const float* ld = part_d + ((size_t)lane * q + j) * k;
    const int32_t* li = part_i + ((size_t)lane * q + j) * k;
    int h = 0;
    for (int r = 0; r < k; ++r) {
        float d = FLT_MAX;
        int32_t i = INT_MAX;
        if (lane < nsplit && h < k) { d = ld[h]; i = li[h]; }
        float bd = d;
        int32_t bi = i;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float od = __shfl_xor(bd, o);
            const int32_t oi = __shfl_xor(bi, o);
            if (before(od, oi, bd, bi)) { bd = od; bi = oi; }
        }
        if (lane == 0) { R_dist[j * k + r] = bd; R_idx[j * k + r] = bi; }
        if (d == bd && i == bi && bi != INT_MAX) ++h;   // row indices are unique, so exactly one lane advances
    }
}

// Running top-k over blocks of database rows: one thread per query merges the list so far (row indices absolute,
// unfilled slots FLT_MAX / INT_MAX) with the list of a block (row indices relative to row0) into `out`.
__global__ void k_topk_merge2(const float* __restrict__ a_d, const int32_t* __restrict__ a_i, int have_a,
                              const float* __restrict__ b_d, const int32_t* __restrict__ b_i, int32_t row0, int64_t q,
                              int k, float* __restrict__ out_d, int32_t* __restrict__ out_i)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= q) return;
    const float* ad = a_d + j * k;
    const int32_t* ai = a_i + j * k;
    const float* bd = b_d + j * k;
    const int32_t* bi = b_i + j * k;
    int ha = 0, hb = 0;
    for (int r = 0; r < k; ++r) {
        float da = FLT_MAX, db = FLT_MAX;
        int32_t ia = INT_MAX, ib = INT_MAX;
        if (have_a && ha < k) { da = ad[ha]; ia = ai[ha]; }
        if (hb < k) { db = bd[hb]; ib = bi[hb]; if (ib != INT_MAX) ib += row0; }
        const bool take_a = before(da, ia, db, ib) || (da == db && ia == ib);
        out_d[j * k + r] = take_a ? da : db;
        out_i[j * k + r] = take_a ? ia : ib;
        if (take_a) ++ha; else ++hb;
    }
}

// Column sums of a block, in fp64: part[split][j] = sum over the rows of the split of tile[r][j] ...
constexpr int kSumSplits = 64;
__global__ __launch_bounds__(256) void k_col_sums_part(const float* __restrict__ tile, int64_t rows, int64_t q, int64_t ldt,
                                                       double* __restrict__ part)
{
    const int lane = threadIdx.x & 63;
    const int64_t j = (int64_t)blockIdx.x * 64 + lane;
    const int split = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int64_t per = (rows + kSumSplits - 1) / kSumSplits;
    const int64_t r0 = split * per, r1 = r0 + per < rows ? r0 + per : rows;
    if (j >= q) return;
    double acc = 0.0;
    int64_t r = r0;
    for (; r + 3 < r1; r += 4) {
        const float x0 = tile[r * ldt + j], x1 = tile[(r + 1) * ldt + j], x2 = tile[(r + 2) * ldt + j], x3 = tile[(r + 3) * ldt + j];
        acc += (double)x0;
        acc += (double)x1;
        acc += (double)x2;
        acc += (double)x3;
    }
    for (; r < r1; ++r) acc += (double)tile[r * ldt + j];
    part[(int64_t)split * q + j] = acc;
}

// ... and sums[j] (+)= the splits' sums in split order: the total does not depend on timing.
__global__ void k_col_sums_add(const double* __restrict__ part, int64_t q, int first, double* __restrict__ sums)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= q) return;
    double acc = first ? 0.0 : sums[j];
    for (int s = 0; s < kSumSplits; ++s) acc += part[(int64_t)s * q + j];
    sums[j] = acc;
}

// Row-wise update for the all-pairs job within one set (lcrwmd_rwmd_self): row r of the tile holds the distances of
// histogram row0 + r to the histograms col_id0 .. col_id0 + q - 1, and R_dist / R_idx hold that row's k nearest so far
// (sorted by (distance, index), unfilled slots FLT_MAX / INT_MAX).  One wavefront per row: the list sits in lanes
// 0 .. k - 1; the row is read 512 values at a time, values that do not beat the list's last entry are skipped, and a
// value that does is inserted by all lanes at once (its place = the number of entries before it; the entries behind
// move up one lane).  Candidates are inserted in column order, so the result does not depend on timing.  row_sum (or
// null): the row's values are added up in fp64 - per lane, then across the lanes in a fixed order - and added to
// row_sum[r].
__global__ __launch_bounds__(256) void k_topk_rows(const float* __restrict__ tile, int64_t rows, int64_t q, int64_t ldt,
                                                   int k, int32_t col_id0, float* __restrict__ R_dist,
                                                   int32_t* __restrict__ R_idx, double* __restrict__ row_sum)
{
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;                       // whole wavefronts leave
    const float* row = tile + r * ldt;
    float ld = FLT_MAX;
    int32_t li = INT_MAX;
    if (lane < k) { ld = R_dist[r * k + lane]; li = R_idx[r * k + lane]; }
    float wd = k > 0 ? __shfl(ld, k - 1) : 0.f;
    int32_t wi = k > 0 ? __shfl(li, k - 1) : 0;
    double acc = 0.0;
    constexpr int UN = 8;
    for (int64_t c0 = 0; c0 < q; c0 += 64 * UN) {
        float v[UN];
#pragma unroll
        for (int t = 0; t < UN; ++t) {
            const int64_t c = c0 + 64 * t + lane;
            v[t] = c < q ? row[c] : FLT_MAX;
        }
#pragma unroll
        for (int t = 0; t < UN; ++t) {
            const int64_t cb = c0 + 64 * t;
            const bool ok = cb + lane < q;
            if (ok) acc += (double)v[t];
            if (k > 0) {
                uint64_t cand = __ballot(ok && before(v[t], col_id0 + (int32_t)(cb + lane), wd, wi));
                while (cand) {
                    const int l = __builtin_ctzll(cand);
                    cand &= cand - 1;
                    const float cv = __shfl(v[t], l);
                    const int32_t ci = col_id0 + (int32_t)(cb + l);
                    const int pos = __builtin_popcountll(__ballot(lane < k && before(ld, li, cv, ci)));
                    if (pos < k) {               // wave-uniform; an earlier insertion of this batch may have closed the gap
                        const float ud = __shfl_up(ld, 1);
                        const int32_t ui = __shfl_up(li, 1);
                        if (lane == pos) { ld = cv; li = ci; }
                        else if (lane > pos) { ld = ud; li = ui; }
                        wd = __shfl(ld, k - 1);
                        wi = __shfl(li, k - 1);
                    }
                }
            }
        }
    }
    if (lane < k) { R_dist[r * k + lane] = ld; R_idx[r * k + lane] = li; }
    if (row_sum) {
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
        if (lane == 0) row_sum[r] += acc;
    }
}

// Scratch of the entry point that allocates nothing: the partial lists live in this array instead of a workspace.
// Every device the library runs on holds its own copy at its own address; host code uses the address obtained by
// topk_static_init, never the array's name.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[kMaxDevices] = {};

}  // namespace

size_t topk_static_bytes() { return kStaticScratchBytes; }

// Called with `device` current (lcrwmd_create): looks up this device's copy of the array once.
hipError_t topk_static_init(int device)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (g_scratch_ptr[device]) return hipSuccess;
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = ptr;
    return hipSuccess;
}

void* topk_static_ptr(int device) { return device >= 0 && device < kMaxDevices ? g_scratch_ptr[device] : nullptr; }

hipError_t launch_topk_merge2(const float* a_d, const int32_t* a_i, bool have_a, const float* b_d, const int32_t* b_i,
                              int64_t row0, int64_t q, int k, float* out_d, int32_t* out_i, hipStream_t s)
{
    if (q <= 0) return hipSuccess;
    k_topk_merge2<<<(unsigned)((q + 63) / 64), 64, 0, s>>>(a_d, a_i, have_a ? 1 : 0, b_d, b_i, (int32_t)row0, q, k, out_d, out_i);
    return hipGetLastError();
}

hipError_t launch_topk_rows(const float* tile, int64_t rows, int64_t q, int64_t ldt, int k, int64_t col_id0, float* R_dist,
                            int32_t* R_idx, double* row_sum, hipStream_t s)
{
    if (rows <= 0 || q <= 0) return hipSuccess;
    if (k < 0 || k > 64 || col_id0 + q > 0x7fffffffLL || (rows + 3) / 4 > 0x7fffffffLL) return hipErrorInvalidValue;
    k_topk_rows<<<(unsigned)((rows + 3) / 4), 256, 0, s>>>(tile, rows, q, ldt, k, (int32_t)col_id0, R_dist, R_idx, row_sum);
    return hipGetLastError();
}

size_t col_sums_bytes(int64_t q) { return (size_t)kSumSplits * (size_t)q * 8 + 256; }

hipError_t launch_col_sums(const float* tile, int64_t rows, int64_t q, int64_t ldt, double* part, bool first, double* sums,
                           hipStream_t s)
{
    if (q <= 0 || rows <= 0) return hipSuccess;
    k_col_sums_part<<<dim3((unsigned)((q + 63) / 64), kSumSplits / 4), 256, 0, s>>>(tile, rows, q, ldt, part);
    k_col_sums_add<<<(unsigned)((q + 255) / 256), 256, 0, s>>>(part, q, first ? 1 : 0, sums);
    return hipGetLastError();
}

size_t topk_bytes(int64_t n, int64_t q, int k)
{
    TopkPlan p = plan_topk(n, q, k, (size_t)-1);
    return p.nsplit > 1 ? (size_t)p.nsplit * (size_t)q * (size_t)k * 8 + 512 : 0;
}

hipError_t launch_topk(const float* D, int64_t n, int64_t q, int64_t ldd, int k, int32_t* R_idx, float* R_dist,
                       void* ws, size_t ws_bytes, hipStream_t s, const float* bound)
{
    if (q <= 0) return hipSuccess;
    Bump b(ws, ws ? ws_bytes : 0);
    TopkPlan p = plan_topk(n, q, k, ws ? ws_bytes - (ws_bytes > 512 ? 512 : ws_bytes) : 0);
    float* pd = R_dist;
    int32_t* pi = R_idx;
    if (p.nsplit > 1) {
        pd = b.take_n<float>((size_t)p.nsplit * q * k);
        pi = b.take_n<int32_t>((size_t)p.nsplit * q * k);
        if (!b.ok) { p.nsplit = 1; p.rows_per_split = n; pd = R_dist; pi = R_idx; }
    }
    const size_t smem = (size_t)k * 256 * 8 + 256 * 4;
    if (smem > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_topk_partial),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    const int64_t grid = p.col_strips * p.nsplit;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    k_topk_partial<<<(unsigned)grid, 256, smem, s>>>(D, n, q, ldd, k, p.rows_per_split, p.col_strips, bound, pd, pi);
    if (p.nsplit > 1) {
        if (q > 0x7fffffffLL) return hipErrorInvalidValue;
        k_topk_merge<<<(unsigned)q, 64, 0, s>>>(pd, pi, q, k, p.nsplit, R_dist, R_idx);
    }
    return hipGetLastError();
}

}  // namespace lcrwmd
