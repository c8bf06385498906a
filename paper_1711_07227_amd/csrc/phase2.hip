// Second phase of LC-RWMD (Sec. IV, Fig. 7): S = X * Z with X the CSR histogram matrix and Z the dense
// matrix of per-word minima, one column per histogram of the other set (many-to-many form).
// Every stored entry (i, p) gathers row p of Z and scales it by the weight, so the work is one fused
// multiply-add per 4-byte load: bandwidth bound.  Lanes run along the columns of Z, so every gather is a
// contiguous row segment; the column and weight of an entry are wave-uniform.
//
// Three write-backs: plain store (D1 of Sec. IV), maximum with what is already in D, and the transposed
// maximum D = max(D1, D2^T) used after the two sets have been swapped.
#include "lcrwmd_internal.h"

namespace lcrwmd {

namespace {

// One batch of up to 64 stored entries of a row, one per lane: column and weight.  Lanes past the end repeat the
// batch's first column with weight 0, so that a batch can be walked in full groups (a repeated row is a valid, finite
// row of Z; it contributes nothing).
struct EntryBatch {
    int cv;
    float xl;
    int cnt;
};

__device__ inline EntryBatch load_entries(int64_t p0, int64_t b, const int32_t* __restrict__ ci, const float* __restrict__ xv, int lane)
{
    EntryBatch e;
    e.cnt = (int)(b - p0 < 64 ? b - p0 : 64);
    e.cv = 0;
    e.xl = 0.f;
    if (lane < e.cnt) { e.cv = ci[p0 + lane]; e.xl = xv[p0 + lane]; }
    // Done here, with every lane active: the values are read across lanes later, also from inside branches that only
    // part of the wavefront takes (a ragged last strip), and a lane must not read a register that was written while
    // the lane it reads from was switched off.
    const int c_first = __builtin_amdgcn_readfirstlane(e.cv);
    if (lane >= e.cnt) e.cv = c_first;
    return e;
}

// acc[t] += sum over the entries of the batch of weight * Z[column][j + t], t < W (full strips: vector gathers).
// UN row segments of Z are requested before the first is used; the gathers of a group are independent of one another.
template <int W, int UN>
__device__ inline void batch_times_strip(const EntryBatch& e, const float* __restrict__ zj, int64_t ldz, float* acc)
{
    typedef float vecw __attribute__((ext_vector_type(W)));
    const int cntu = (e.cnt + UN - 1) / UN * UN;          // cnt <= 64 and UN divides 64
    for (int u = 0; u < cntu; u += UN) {
        vecw z[UN];
#pragma unroll
        for (int k = 0; k < UN; ++k)
            z[k] = *reinterpret_cast<const vecw*>(zj + (int64_t)__builtin_amdgcn_readlane(e.cv, u + k) * ldz);
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            const float x = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, e.xl), u + k));
#pragma unroll
            for (int t = 0; t < W; ++t) acc[t] = fmaf(x, z[k][t], acc[t]);
        }
    }
}

// acc[t] = sum over the stored entries p in [a, b) of xv[p] * Z[ci[p]][j + t], t < W, for this lane's columns
// j .. j + W - 1 (a, b wave-uniform).  `first` holds the entries [a, a + 64) already (requested by the caller while it
// was busy with the row before: a row costs the round trips of its gathers only).
template <int W>
__device__ inline void row_times_strip(int64_t a, int64_t b, EntryBatch first, const int32_t* __restrict__ ci,
                                       const float* __restrict__ xv, const float* __restrict__ Z, int64_t ldz, int64_t ncols,
                                       int64_t j, int lane, float* acc)
{
#pragma unroll
    for (int t = 0; t < W; ++t) acc[t] = 0.f;
    const bool full = j + W - 1 < ncols;
    const float* zj = Z + j;
    EntryBatch e = first;
    for (int64_t p0 = a; p0 < b; p0 += 64) {
        if (p0 > a) e = load_entries(p0, b, ci, xv, lane);
        if (full) {
            batch_times_strip<W, 8>(e, zj, ldz, acc);
        } else {
            for (int u = 0; u < e.cnt; ++u) {
                const float* zr = zj + (int64_t)__builtin_amdgcn_readlane(e.cv, u) * ldz;
                const float x = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, e.xl), u));
#pragma unroll
                for (int t = 0; t < W; ++t)
                    if (j + t < ncols) acc[t] = fmaf(x, zr[t], acc[t]);
            }
        }
    }
}

__device__ inline int64_t uniform_i64(int64_t x)
{
    return (int64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)x) | ((int64_t)__builtin_amdgcn_readfirstlane((int)(x >> 32)) << 32);
}

// Which item of a strip-major list of `total` work items this workgroup takes, or -1.  The part has eight XCDs, each
// with an L2 of its own, and hands workgroup b to XCD b mod 8: item k of XCD x is item x * per + k of the list, so an
// XCD works through one contiguous eighth of it - its own strips of columns - and its L2 holds segments of Z's rows
// that no other XCD asks for.  (With the whole chip on one strip at a time every L2 fetched every segment: eight
// copies of the same lines, an eighth of the cache.)  Any other assignment of workgroups to XCDs is still correct:
// every item is taken exactly once.  per = ceil(total / 8), grid = 8 * per.
constexpr int kXcds = 8;
__device__ inline int64_t xcd_item(int64_t per, int64_t total)
{
    const int64_t x = blockIdx.x % kXcds, k = blockIdx.x / kXcds;
    const int64_t it = x * per + k;
    return it < total ? it : -1;
}

// One wavefront per (RPW consecutive rows, strip of 64*W columns); W = 4 uses 16-byte gathers, W = 2 8-byte ones.
// Units are ordered strip-major and dealt to the XCDs in contiguous ranges (xcd_item), so an XCD works on one strip of
// columns at a time: its strip of Z (rows of 256 W bytes) is what has to stay in its L2, not the full rows.  The row
// pointers of a unit are fetched in one load and the entries of the next row are requested before the gathers of the
// current one.
constexpr int RPW = 4;
template <int W, int COMBINE>
__global__ __launch_bounds__(256) void k_spmm_rows(const int64_t* __restrict__ rp, const int32_t* __restrict__ ci,
                                                   const float* __restrict__ xv, int64_t rows,
                                                   const float* __restrict__ Z, int64_t ldz, int64_t ncols,
                                                   float* __restrict__ D, int64_t ldd, int64_t strips, int64_t row_units,
                                                   int64_t per, int64_t total)
{
    const int lane = threadIdx.x & 63;
    const int64_t item = xcd_item(per, total);
    if (item < 0) return;
    const int64_t unit = item * 4 + (threadIdx.x >> 6);
    const int64_t strip = unit / row_units;
    const int64_t i0 = (unit - strip * row_units) * RPW;
    if (strip >= strips) return;
    const int64_t j = strip * (64 * W) + (int64_t)lane * W;
    // row bounds are wave-uniform: keep them scalar so that the loop control and the row addresses of Z are scalar too
    const int nr = (int)(rows - i0 < RPW ? rows - i0 : RPW);
    const int64_t mine = rp[i0 + (lane <= nr ? lane : nr)];
    int64_t bound[RPW + 1];
#pragma unroll
    for (int r = 0; r <= RPW; ++r) bound[r] = uniform_i64(__shfl(mine, r < nr ? r : nr));
    EntryBatch next = load_entries(bound[0], bound[1], ci, xv, lane);
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        if (r < nr) {
            const EntryBatch cur = next;
            if (r + 1 < nr) next = load_entries(bound[r + 1], bound[r + 2], ci, xv, lane);
            float acc[W];
            row_times_strip<W>(bound[r], bound[r + 1], cur, ci, xv, Z, ldz, ncols, j, lane, acc);
#pragma unroll
            for (int t = 0; t < W; ++t) {
                if (j + t < ncols) {
                    float* d = D + (i0 + r) * ldd + j + t;
                    if (COMBINE == 0) *d = acc[t];
                    else *d = fmaxf(*d, acc[t]);
                }
            }
        }
    }
}

// Transposed maximum: X has `rows` histograms (the queries after the swap), Z has ncols columns (the
// database rows of the current batch); D[c * ldd + r] = max(D[c * ldd + r], S[r][c]).
// A workgroup computes a 32 (rows of X) x 64 (columns) tile of S with lanes along the columns, then
// turns it through LDS so that the read-modify-write of D is along D's rows.
constexpr int TR = 32, TC = 64;

__global__ __launch_bounds__(256) void k_spmm_tmax(const int64_t* __restrict__ rp, const int32_t* __restrict__ ci,
                                                   const float* __restrict__ xv, int64_t rows,
                                                   const float* __restrict__ Z, int64_t ldz, int64_t ncols,
                                                   float* __restrict__ D, int64_t ldd, int64_t row_tiles)
{
    __shared__ float tile[TR][TC + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // row tiles vary fastest: the workgroups that share a strip of Z columns run together
    const int64_t ct = blockIdx.x / row_tiles;
    const int64_t rt = blockIdx.x - ct * row_tiles;
    const int64_t r0 = rt * TR, c0 = ct * TC;
    const int64_t c = c0 + lane;
    const bool c_ok = c < ncols;
    const int64_t cc = c_ok ? c : ncols - 1;

    for (int k = 0; k < TR / 4; ++k) {
        const int rr = wave * (TR / 4) + k;
        const int64_t r = r0 + rr;
        float acc = 0.f;
        if (r < rows) {
            const int64_t a = rp[r], b = rp[r + 1];
            int64_t p = a;
            for (; p + 3 < b; p += 4) {
                const float z0 = Z[(int64_t)ci[p] * ldz + cc], z1 = Z[(int64_t)ci[p + 1] * ldz + cc];
                const float z2 = Z[(int64_t)ci[p + 2] * ldz + cc], z3 = Z[(int64_t)ci[p + 3] * ldz + cc];
                acc = fmaf(xv[p], z0, acc);
                acc = fmaf(xv[p + 1], z1, acc);
                acc = fmaf(xv[p + 2], z2, acc);
                acc = fmaf(xv[p + 3], z3, acc);
            }
            for (; p < b; ++p) acc = fmaf(xv[p], Z[(int64_t)ci[p] * ldz + cc], acc);
        }
        tile[rr][lane] = acc;
    }
    __syncthreads();
    // thread -> (column of the tile = row of D, 32 consecutive entries of that row)
    const int tr = threadIdx.x & (TR - 1);
    for (int tc = threadIdx.x / TR; tc < TC; tc += 256 / TR) {
        const int64_t dr = c0 + tc, dc = r0 + tr;
        if (dr < ncols && dc < rows) {
            float* d = D + dr * ldd + dc;
            *d = fmaxf(*d, tile[tr][tc]);
        }
    }
}

// Transposed maximum, wide form: a workgroup computes a 32 (rows of X) x 256 (columns) tile of S, every wavefront
// 8 rows with 16-byte gathers exactly as k_spmm_rows does, and turns the tile through LDS so that the
// read-modify-write of D runs along D's rows (32 consecutive floats = one 128-byte line per column of the tile).
// Needs 16-byte aligned rows of Z.  Row tiles vary fastest and the list of tiles is dealt to the XCDs in contiguous
// ranges (xcd_item), so the workgroups that share a strip of columns of Z share an L2.
constexpr int WR = 32, WC = 256;

__global__ __launch_bounds__(256) void k_spmm_tmax_wide(const int64_t* __restrict__ rp, const int32_t* __restrict__ ci,
                                                        const float* __restrict__ xv, int64_t rows,
                                                        const float* __restrict__ Z, int64_t ldz, int64_t ncols,
                                                        float* __restrict__ D, int64_t ldd, int64_t row_tiles,
                                                        int64_t per, int64_t total)
{
    __shared__ float tile[WR][WC + 1];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t item = xcd_item(per, total);
    if (item < 0) return;                       // the whole workgroup: no barrier is left waiting
    const int64_t ct = item / row_tiles;
    const int64_t rt = item - ct * row_tiles;
    const int64_t r0 = rt * WR, c0 = ct * WC;
    const int64_t j = c0 + (int64_t)lane * 4;

    // this wavefront's WR / 4 rows: their bounds in one load, the entries of the next row requested before the gathers of
    // the current one
    constexpr int NR = WR / 4;
    const int64_t rw = r0 + wave * NR;
    const int nr = (int)(rows - rw < NR ? (rows - rw > 0 ? rows - rw : 0) : NR);
    int64_t bound[NR + 1];
    {
        const int64_t mine = nr > 0 ? rp[rw + (lane <= nr ? lane : nr)] : 0;
#pragma unroll
        for (int r = 0; r <= NR; ++r) bound[r] = uniform_i64(__shfl(mine, r < nr ? r : nr));
    }
    EntryBatch next = load_entries(bound[0], bound[1], ci, xv, lane);
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        const int rr = wave * NR + k;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        if (k < nr) {
            const EntryBatch cur = next;
            if (k + 1 < nr) next = load_entries(bound[k + 1], bound[k + 2], ci, xv, lane);
            row_times_strip<4>(bound[k], bound[k + 1], cur, ci, xv, Z, ldz, ncols, j, lane, acc);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) tile[rr][4 * lane + t] = acc[t];
    }
    __syncthreads();
    // thread -> (row of the tile = position along D's row, column of the tile = row of D)
    const int tr = threadIdx.x & (WR - 1);
    for (int tc = threadIdx.x / WR; tc < WC; tc += 256 / WR) {
        const int64_t dr = c0 + tc, dc = r0 + tr;
        if (dr < ncols && dc < rows) {
            float* d = D + dr * ldd + dc;
            *d = fmaxf(*d, tile[tr][tc]);
        }
    }
}

}  // namespace

hipError_t launch_spmm(const int64_t* rp, const int32_t* ci, const float* xv, int64_t rows, const float* Z,
                       int64_t ldz, int64_t zrows, int64_t ncols, float* D, int64_t ldd, int combine, hipStream_t s)
{
    (void)zrows;
    if (rows <= 0 || ncols <= 0) return hipSuccess;
    if (combine == 2 && (ldz % 4 == 0) && (((uintptr_t)Z & 15) == 0) && ncols >= 128) {
        const int64_t row_tiles = (rows + WR - 1) / WR, col_tiles = (ncols + WC - 1) / WC;
        const int64_t total = row_tiles * col_tiles, per = (total + kXcds - 1) / kXcds, grid = per * kXcds;
        if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
        k_spmm_tmax_wide<<<(unsigned)grid, 256, 0, s>>>(rp, ci, xv, rows, Z, ldz, ncols, D, ldd, row_tiles, per, total);
        return hipGetLastError();
    }
    if (combine == 2) {
        const int64_t row_tiles = (rows + TR - 1) / TR, col_tiles = (ncols + TC - 1) / TC;
        const int64_t grid = row_tiles * col_tiles;
        if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
        k_spmm_tmax<<<(unsigned)grid, 256, 0, s>>>(rp, ci, xv, rows, Z, ldz, ncols, D, ldd, row_tiles);
        return hipGetLastError();
    }
    // strip width: 16-byte gathers need 16-byte aligned rows of Z; narrower strips keep more rows of the strip in cache
    int W = 1;
    if ((ldz % 4 == 0) && (((uintptr_t)Z & 15) == 0) && ncols >= 256) W = 4;
    else if ((ldz % 2 == 0) && (((uintptr_t)Z & 7) == 0) && ncols >= 128) W = 2;
    const int64_t strips = (ncols + 64 * W - 1) / (64 * W);
    const int64_t row_units = (rows + RPW - 1) / RPW;
    const int64_t total = (row_units * strips + 3) / 4, per = (total + kXcds - 1) / kXcds, grid = per * kXcds;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
#define LAUNCH_ROWS(WW, CC) \
    k_spmm_rows<WW, CC><<<(unsigned)grid, 256, 0, s>>>(rp, ci, xv, rows, Z, ldz, ncols, D, ldd, strips, row_units, per, total)
    if (W == 4) { if (combine == 0) LAUNCH_ROWS(4, 0); else LAUNCH_ROWS(4, 1); }
    else if (W == 2) { if (combine == 0) LAUNCH_ROWS(2, 0); else LAUNCH_ROWS(2, 1); }
    else { if (combine == 0) LAUNCH_ROWS(1, 0); else LAUNCH_ROWS(1, 1); }
#undef LAUNCH_ROWS
    return hipGetLastError();
}

}  // namespace lcrwmd
