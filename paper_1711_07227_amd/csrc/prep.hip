// Support kernels of the LC-RWMD path: squared row norms of E, vocabulary reduction
// (Sec. IV: words that do not occur in the resident set are dropped), the padded token list
// of a batch of histograms (the stacked T matrix of the many-to-many form, kept as word ids),
// the exact-zero fix-up for words that occur in the histogram itself, and CSR validation.
#include "lcrwmd_internal.h"

namespace lcrwmd {

namespace {

constexpr int kScanThreads = 1024;

__global__ void k_fill_i32(int32_t* p, int64_t n, int32_t value)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = value;
}

// One wavefront per row: normE[w] = sum_t E[w][t]^2 in fp32.
__global__ __launch_bounds__(256) void k_row_norms_f32(const float* __restrict__ E, int64_t v, int32_t m,
                                                       int64_t ld, float* __restrict__ normE)
{
    const int lane = threadIdx.x & 63;
    int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= v) return;
    const float* row = E + w * ld;
    float s = 0.f;
    for (int t = lane; t < m; t += 64) { float x = row[t]; s = fmaf(x, x, s); }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) normE[w] = s;
}

// One wavefront per row: a copy of E with `pitch` floats per row, zeros beyond column m, and the squared norms.
__global__ __launch_bounds__(256) void k_pack_f32(const float* __restrict__ E, int64_t v, int32_t m, int64_t ld,
                                                  int32_t pitch, float* __restrict__ packed, float* __restrict__ normE)
{
    const int lane = threadIdx.x & 63;
    int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= v) return;
    const float* row = E + w * ld;
    float* out = packed + w * pitch;
    float s = 0.f;
    for (int t = lane; t < pitch; t += 64) {
        const float x = t < m ? row[t] : 0.f;
        out[t] = x;
        s = fmaf(x, x, s);
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) normE[w] = s;
}

// fp32 copy (pitch m) of bf16-valued embeddings: bf16 storage widened, or fp32 storage rounded to bf16 (nearest even).
__global__ void k_widen_bf16(const void* __restrict__ E, int is_bf16, int64_t v, int32_t m, int64_t ld, float* __restrict__ out)
{
    const int64_t total = v * m;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t w = e / m;
        const int32_t t = (int32_t)(e - w * m);
        uint32_t bits;
        if (is_bf16) {
            bits = (uint32_t)reinterpret_cast<const uint16_t*>(E)[w * ld + t] << 16;
        } else {
            const uint32_t u = __float_as_uint(reinterpret_cast<const float*>(E)[w * ld + t]);
            bits = (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
        }
        out[e] = __uint_as_float(bits);
    }
}

__global__ void k_iota_i32(int32_t* p, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = (int32_t)i;
}

__global__ void k_mark_words(const int32_t* __restrict__ col_idx, int64_t nnz, int32_t* __restrict__ flags)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < nnz; i += stride) flags[col_idx[i]] = 1;   // benign race: every writer stores 1
}

// Exclusive block scan helper: returns the exclusive prefix of x over the block and the block total.
__device__ inline int32_t block_exclusive_scan(int32_t x, int32_t* wave_sums, int32_t& total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t incl = x;
    for (int o = 1; o < 64; o <<= 1) {
        int32_t y = __shfl_up(incl, o);
        if (lane >= o) incl += y;
    }
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t run = 0;
        for (int k = 0; k < kScanThreads / 64; ++k) { int32_t t = wave_sums[k]; wave_sums[k] = run; run += t; }
        wave_sums[kScanThreads / 64] = run;
    }
    __syncthreads();
    int32_t excl = wave_sums[wave] + incl - x;
    total = wave_sums[kScanThreads / 64];
    __syncthreads();   // wave_sums is reused by the next strip
    return excl;
}

// Single workgroup: stream compaction of the flagged words, in increasing word id.
__global__ __launch_bounds__(kScanThreads) void k_compact_words(const int32_t* __restrict__ flags, int64_t v,
                                                                int32_t* __restrict__ list,
                                                                int32_t* __restrict__ map,
                                                                int32_t* __restrict__ count)
{
    __shared__ int32_t wave_sums[kScanThreads / 64 + 1];
    int32_t carry = 0;
    for (int64_t base = 0; base < v; base += kScanThreads) {
        int64_t w = base + threadIdx.x;
        int32_t f = (w < v && flags[w] != 0) ? 1 : 0;
        int32_t total;
        int32_t pos = carry + block_exclusive_scan(f, wave_sums, total);
        if (w < v) {
            if (f) list[pos] = (int32_t)w;
            if (map) map[w] = f ? pos : -1;
        }
        carry += total;
    }
    if (threadIdx.x == 0) *count = carry;
}

__global__ void k_remap_cols(const int32_t* __restrict__ col_idx, int64_t nnz, const int32_t* __restrict__ map,
                             int32_t* __restrict__ out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < nnz; i += stride) out[i] = map[col_idx[i]];
}

// Single workgroup: pofs[s] = sum_{r<s} len_r rounded up to the group size; pofs[nseg] = padded total.
__global__ __launch_bounds__(kScanThreads) void k_seg_offsets(const int64_t* __restrict__ rp, int64_t nseg,
                                                              int32_t* __restrict__ pofs, int group)
{
    __shared__ int32_t wave_sums[kScanThreads / 64 + 1];
    int32_t carry = 0;
    for (int64_t base = 0; base < nseg; base += kScanThreads) {
        int64_t s = base + threadIdx.x;
        int32_t len = 0;
        if (s < nseg) {
            int64_t l = rp[s + 1] - rp[s];
            if (l < 0) l = 0;
            len = (int32_t)((l + (group - 1)) & ~(int64_t)(group - 1));
        }
        int32_t total;
        int32_t pos = carry + block_exclusive_scan(len, wave_sums, total);
        if (s < nseg) pofs[s] = pos;
        carry += total;
    }
    if (threadIdx.x == 0) pofs[nseg] = carry;
}

// Largest s in [0, nseg] with pofs[s] <= x (pofs is non-decreasing, pofs[0] == 0 <= x).
__device__ inline int32_t last_le(const int32_t* pofs, int32_t nseg, int32_t x)
{
    int32_t lo = 0, hi = nseg + 1;   // invariant: pofs[lo] <= x, (hi == nseg+1 or pofs[hi] > x)
    while (hi - lo > 1) {
        int32_t mid = lo + ((hi - lo) >> 1);
        if (pofs[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// One thread per group of padded tokens.
__global__ void k_fill_tokens(const int64_t* __restrict__ rp, const int32_t* __restrict__ col_idx, int32_t nseg,
                              const int32_t* __restrict__ pofs, const float* __restrict__ normE,
                              int32_t* __restrict__ tok_ids, float* __restrict__ tok_hn,
                              int32_t* __restrict__ grp_seg, int64_t ngroups_alloc, int group)
{
    int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= ngroups_alloc) return;
    const int32_t total = pofs[nseg];
    const int64_t start = g * group;
    if (start >= total) {
        grp_seg[g] = -1;
        for (int t = 0; t < group; ++t) { tok_ids[start + t] = 0; tok_hn[start + t] = 0.f; }
        return;
    }
    const int32_t seg = last_le(pofs, nseg, (int32_t)start);   // equal offsets: the last one is the non-empty one
    const int64_t base = rp[seg];
    const int64_t len = rp[seg + 1] - base;
    const int64_t pos0 = start - pofs[seg];
    grp_seg[g] = seg;
    for (int t = 0; t < group; ++t) {
        int64_t pos = pos0 + t;
        if (pos > len - 1) pos = len - 1;                       // pad by repeating the last word
        int32_t id = col_idx[base + pos];
        tok_ids[start + t] = id;
        tok_hn[start + t] = -0.5f * normE[id];
    }
}

// chunk_seg[c] = first segment whose padded offset is >= c * chunk_tokens (nseg when there is none).
__global__ void k_chunk_bounds(const int32_t* __restrict__ pofs, int32_t nseg, int32_t chunk_tokens,
                               int32_t nchunks, int32_t* __restrict__ chunk_seg)
{
    int32_t c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c > nchunks) return;
    int64_t x = (int64_t)c * chunk_tokens;
    int32_t lo = 0, hi = nseg;      // answer in [0, nseg]
    while (lo < hi) {
        int32_t mid = lo + ((hi - lo) >> 1);
        if ((int64_t)pofs[mid] >= x) hi = mid; else lo = mid + 1;
    }
    chunk_seg[c] = lo;
}

// One wavefront per histogram.  bits (or null): the contraction kernel's map of close pairs (see k_redo_close_bits);
// the entries set to exactly 0 here are taken out of it, so that the pass over the map is left with the pairs of
// different words only - on ordinary embeddings nothing at all.
__global__ __launch_bounds__(256) void k_zero_matches(const int64_t* __restrict__ rp,
                                                      const int32_t* __restrict__ col_idx, int64_t nseg,
                                                      const int32_t* __restrict__ map, float* __restrict__ Z,
                                                      int64_t ldz, uint64_t* __restrict__ bits, int64_t pitch, int slice_words)
{
    const int lane = threadIdx.x & 63;
    int64_t seg = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (seg >= nseg) return;
    for (int64_t p = rp[seg] + lane; p < rp[seg + 1]; p += 64) {
        int32_t w = col_idx[p];
        int32_t row = map ? map[w] : w;
        if (row >= 0) {
            Z[(int64_t)row * ldz + seg] = 0.f;
            if (bits) {
                const int b = row % slice_words;
                // 32-position slices carry every bit twice (both lane halves of the wavefront that wrote them)
                const unsigned long long gone = slice_words == 32 ? ((1ull << b) | (1ull << (b + 32))) : (1ull << b);
                atomicAnd(reinterpret_cast<unsigned long long*>(bits + seg * pitch + row / slice_words), ~gone);
            }
        }
    }
}

// Where a word and a word of the histogram lie close together, the squared distance the contraction delivers,
// |x|^2 + |y|^2 - 2 x.y, is a small difference of large numbers: its absolute error is a few 1e-6 (|x|^2 + |y|^2), so
// the relative error of the distance passes 1e-4 once d^2 falls below a few percent of the squared norms - and the
// minimum of the first phase picks exactly those entries.  This pass re-evaluates every entry of Z whose square is
// below a quarter of the word's squared norm from coordinate differences, sum_t (x_t - y_t)^2, whose error is relative
// to d^2 itself.  (An entry above that threshold came from a d^2 >= (|x|^2 + |y|^2) / 8 or so - two vectors whose
// norms differ by more than a factor 1.5 are further apart than half the shorter one - where the expansion is good
// to 1e-5.)  The minimum of the exact distances is taken over all words of the histogram: the expansion's ranking of
// near neighbours is not trusted either.  An entry whose word itself occurs in the histogram is recognised by a
// binary search in the sorted row and set to exactly 0 (k_zero_matches, where it ran before, has done so already).
//
// One wavefront per row of Z and strip of columns: 64 entries are tested at a time (one coalesced load); the flagged
// ones are then redone one after the other by the whole wavefront, lanes along the embedding dimension.  On embeddings
// without close pairs this is one read of Z.
constexpr int kRedoCols = 1024;      // columns per wavefront: four 16-byte loads per lane, all in flight together

template <bool BF16>
__device__ inline float emb_value(const void* E, int64_t idx)
{
    if (BF16) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(E)[idx] << 16);
    return reinterpret_cast<const float*>(E)[idx];
}

// VEC: rows of Z are 16-byte aligned (pitch a multiple of 4, base aligned): lanes read float4; otherwise scalars.
template <bool BF16, bool VEC>
__global__ __launch_bounds__(256) void k_redo_close(const void* __restrict__ E, int64_t ld, int32_t m,
                                                    const float* __restrict__ normE, const int32_t* __restrict__ voc_rows,
                                                    int64_t nvoc, const int64_t* __restrict__ rp,
                                                    const int32_t* __restrict__ ci, int64_t nseg, float* __restrict__ Z,
                                                    int64_t ldz, int64_t strips)
{
    const int lane = threadIdx.x & 63;
    const int64_t unit = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t pos = unit / strips;
    if (pos >= nvoc) return;
    const int64_t strip = unit - pos * strips;
    const int32_t w = voc_rows ? voc_rows[pos] : (int32_t)pos;
    const float limit = 0.25f * normE[w];
    float* zrow = Z + pos * ldz;
    // element e of this lane: column j0 + 256 * (e / 4) + 4 * lane + e % 4 (VEC) or j0 + 64 * e + lane
    const int64_t j0 = strip * kRedoCols;
    float z[16];
    if (VEC) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int64_t j = j0 + 256 * b + 4 * lane;
            float4 x = make_float4(1e30f, 1e30f, 1e30f, 1e30f);
            if (j + 3 < nseg) x = *reinterpret_cast<const float4*>(zrow + j);
            else {
                if (j < nseg) x.x = zrow[j];
                if (j + 1 < nseg) x.y = zrow[j + 1];
                if (j + 2 < nseg) x.z = zrow[j + 2];
            }
            z[4 * b] = x.x; z[4 * b + 1] = x.y; z[4 * b + 2] = x.z; z[4 * b + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int64_t j = j0 + 64 * e + lane;
            z[e] = j < nseg ? zrow[j] : 1e30f;
        }
    }
    bool any = false;
#pragma unroll
    for (int e = 0; e < 16; ++e) any |= z[e] * z[e] < limit;
    if (!__any(any)) return;

#pragma unroll 1
    for (int e = 0; e < 16; ++e) {
        const int64_t j = VEC ? j0 + 256 * (e >> 2) + 4 * lane + (e & 3) : j0 + 64 * e + lane;
        float ze = z[0];
#pragma unroll
        for (int t = 1; t < 16; ++t) ze = e == t ? z[t] : ze;
        bool redo = j < nseg && ze * ze < limit;
        if (redo) {
            // the word itself in the histogram?  (rows are sorted)  Then the distance is exactly 0.
            int64_t lo = rp[j], hi = rp[j + 1];
            while (lo < hi) {
                const int64_t mid = lo + ((hi - lo) >> 1);
                if (ci[mid] < w) lo = mid + 1; else hi = mid;
            }
            if (lo < rp[j + 1] && ci[lo] == w) {
                if (ze != 0.f) zrow[j] = 0.f;
                redo = false;
            }
        }
        uint64_t todo = __ballot(redo);
        while (todo) {
            const int l = __builtin_ctzll(todo);
            todo &= todo - 1;
            const int64_t jj = __builtin_amdgcn_readlane((int)(j - j0), l) + j0;
            const int64_t a = rp[jj], b = rp[jj + 1];
            float best = 3.0e38f;
            for (int64_t t = a; t < b; ++t) {
                const int32_t c = ci[t];
                float s = 0.f;
                for (int32_t k = lane; k < m; k += 64) {
                    const float d = emb_value<BF16>(E, (int64_t)w * ld + k) - emb_value<BF16>(E, (int64_t)c * ld + k);
                    s = fmaf(d, d, s);
                }
                for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
                best = fminf(best, s);
            }
            if (lane == l) zrow[j] = sqrtf(best);
        }
    }
}

// The second look driven by the contraction kernel's map of close pairs: one thread per 64-bit word of the map.  A
// set bit is either the word itself in the histogram (binary search in the sorted row: the entry is exactly 0) or a
// pair of different words that lie close: those are redone from coordinate differences by the whole wavefront, one
// after the other, lanes along the embedding dimension.
template <bool BF16>
__global__ __launch_bounds__(256) void k_redo_close_bits(const void* __restrict__ E, int64_t ld, int32_t m,
                                                         const int32_t* __restrict__ voc_rows, int64_t nvoc,
                                                         const int64_t* __restrict__ rp, const int32_t* __restrict__ ci,
                                                         int64_t nseg, float* __restrict__ Z, int64_t ldz,
                                                         const uint64_t* __restrict__ bits, int64_t pitch, int slice_words)
{
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t j = t / pitch, slice = t - j * pitch;
    uint64_t mine = j < nseg ? bits[t] : 0;
    if (slice_words == 32) mine &= 0xffffffffull;                 // both lane halves hold the same 32 positions
    if (!__any(mine != 0)) return;
    while (__any(mine != 0)) {
        // this lane's next candidate
        int64_t pos = -1;
        int32_t w = 0;
        bool redo = false;
        if (mine) {
            const int bit = __builtin_ctzll(mine);
            mine &= mine - 1;
            pos = slice * slice_words + bit;
            if (pos < nvoc) {
                w = voc_rows ? voc_rows[pos] : (int32_t)pos;
                int64_t lo = rp[j], hi = rp[j + 1];
                while (lo < hi) {
                    const int64_t mid = lo + ((hi - lo) >> 1);
                    if (ci[mid] < w) lo = mid + 1; else hi = mid;
                }
                if (lo < rp[j + 1] && ci[lo] == w) Z[pos * ldz + j] = 0.f;
                else redo = true;
            }
        }
        uint64_t todo = __ballot(redo);
        while (todo) {
            const int l = __builtin_ctzll(todo);
            todo &= todo - 1;
            const int32_t ww = __builtin_amdgcn_readlane(w, l);
            const int64_t jj = __shfl(j, l);
            const int64_t a = rp[jj], b = rp[jj + 1];
            float best = 3.0e38f;
            for (int64_t e = a; e < b; ++e) {
                const int32_t c = ci[e];
                float sum = 0.f;
                for (int32_t k = lane; k < m; k += 64) {
                    const float d = emb_value<BF16>(E, (int64_t)ww * ld + k) - emb_value<BF16>(E, (int64_t)c * ld + k);
                    sum = fmaf(d, d, sum);
                }
                for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
                best = fminf(best, sum);
            }
            if (lane == l) Z[pos * ldz + j] = sqrtf(best);
        }
    }
}

__global__ void k_validate_csr(const int64_t* __restrict__ rp, const int32_t* __restrict__ col_idx,
                               const float* __restrict__ val, int64_t rows, int64_t cols, int64_t nnz,
                               int32_t* __restrict__ status)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0 && (rp[0] != 0 || rp[rows] != nnz)) atomicMax(status, (int32_t)LCRWMD_EBADCSR);
    if (i >= rows) return;
    int64_t a = rp[i], b = rp[i + 1];
    if (a < 0 || b > nnz || b < a) { atomicMax(status, (int32_t)LCRWMD_EBADCSR); return; }
    if (b == a) { atomicMax(status, (int32_t)LCRWMD_EEMPTYDOC); return; }
    int32_t prev = -1;
    bool bad = false;
    for (int64_t p = a; p < b; ++p) {
        int32_t c = col_idx[p];
        if (c <= prev || c >= cols) bad = true;
        if (val && !(val[p] > 0.f)) bad = true;
        prev = c;
    }
    if (bad) atomicMax(status, (int32_t)LCRWMD_EBADCSR);   // EEMPTYDOC (3) outranks EBADCSR (2) only in number
}

inline int grid_for(int64_t n, int threads, int cap = 1 << 20)
{
    int64_t g = (n + threads - 1) / threads;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace

hipError_t launch_fill_i32(int32_t* p, int64_t n, int32_t value, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    k_fill_i32<<<grid_for(n, 256, 8192), 256, 0, s>>>(p, n, value);
    return hipGetLastError();
}

hipError_t launch_iota_i32(int32_t* p, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    k_iota_i32<<<grid_for(n, 256, 8192), 256, 0, s>>>(p, n);
    return hipGetLastError();
}

hipError_t launch_row_norms_f32(const float* E, int64_t v, int32_t m, int64_t ld, float* normE, hipStream_t s)
{
    if (v <= 0) return hipSuccess;
    k_row_norms_f32<<<(unsigned)((v + 3) / 4), 256, 0, s>>>(E, v, m, ld, normE);
    return hipGetLastError();
}

hipError_t launch_pack_f32(const float* E, int64_t v, int32_t m, int64_t ld, int32_t pitch, float* packed, float* normE,
                           hipStream_t s)
{
    if (v <= 0) return hipSuccess;
    k_pack_f32<<<(unsigned)((v + 3) / 4), 256, 0, s>>>(E, v, m, ld, pitch, packed, normE);
    return hipGetLastError();
}

hipError_t launch_widen_bf16(const void* E, lcrwmd_dtype dtype, int64_t v, int32_t m, int64_t ld, float* out, hipStream_t s)
{
    if (v <= 0) return hipSuccess;
    k_widen_bf16<<<grid_for(v * m, 256, 16384), 256, 0, s>>>(E, dtype == LCRWMD_BF16 ? 1 : 0, v, m, ld, out);
    return hipGetLastError();
}

hipError_t launch_mark_words(const int32_t* col_idx, int64_t nnz, int32_t* flags, hipStream_t s)
{
    if (nnz <= 0) return hipSuccess;
    k_mark_words<<<grid_for(nnz, 256, 8192), 256, 0, s>>>(col_idx, nnz, flags);
    return hipGetLastError();
}

hipError_t launch_compact_words(const int32_t* flags, int64_t v, int32_t* list, int32_t* map, int32_t* count,
                                hipStream_t s)
{
    k_compact_words<<<1, kScanThreads, 0, s>>>(flags, v, list, map, count);
    return hipGetLastError();
}

hipError_t launch_remap_cols(const int32_t* col_idx, int64_t nnz, const int32_t* map, int32_t* out, hipStream_t s)
{
    if (nnz <= 0) return hipSuccess;
    k_remap_cols<<<grid_for(nnz, 256, 8192), 256, 0, s>>>(col_idx, nnz, map, out);
    return hipGetLastError();
}

size_t token_plan_bytes(int64_t nseg, int64_t nnz_batch)
{
    Bump b((void*)256, (size_t)1 << 60);   // dry run: only the byte count matters
    TokenPlan tp;
    carve_token_plan(b, tp, nseg, nnz_batch, 1);
    return b.used + 256;
}

bool carve_token_plan(Bump& b, TokenPlan& tp, int64_t nseg, int64_t nnz_batch, int64_t nvoc_tiles, int64_t padded_exact,
                      int group, int max_chunk_tiles)
{
    tp.nseg = nseg;
    tp.group = group;
    tp.tok_bound = nnz_batch + (kGroup - 1) * nseg;
    tp.tok_alloc = ((tp.tok_bound + kTileTokens - 1) / kTileTokens + 1) * kTileTokens;
    // Aim at a few thousand workgroups (vocabulary tiles x chunks) so that 256 CUs stay busy and the
    // tail is short, while each chunk still spans many token tiles.
    int64_t want_chunks = (4096 + nvoc_tiles - 1) / (nvoc_tiles > 0 ? nvoc_tiles : 1);
    if (want_chunks < 1) want_chunks = 1;
    int64_t ct = (tp.tok_bound + want_chunks - 1) / want_chunks;
    ct = ((ct + kTileTokens - 1) / kTileTokens) * kTileTokens;
    if (ct < 4 * kTileTokens) ct = 4 * kTileTokens;
    if (ct > max_chunk_tiles * kTileTokens) ct = (int64_t)max_chunk_tiles * kTileTokens;
    tp.chunk_tokens = (int32_t)ct;
    const int64_t tok_for_chunks = padded_exact >= 0 ? padded_exact : tp.tok_bound;
    tp.nchunks = (int32_t)((tok_for_chunks + ct - 1) / ct);
    if (tp.nchunks < 1) tp.nchunks = 1;
    // the dry run used for sizing passes nvoc_tiles = 1, which yields the largest chunk count it can
    // ever need only if chunks never get smaller than the floor: size for the floor.
    int64_t chunks_alloc = (tp.tok_bound + 4 * kTileTokens - 1) / (4 * kTileTokens) + 2;
    tp.pofs = b.take_n<int32_t>((size_t)nseg + 1);
    tp.tok_ids = b.take_n<int32_t>((size_t)tp.tok_alloc);
    tp.tok_hn = b.take_n<float>((size_t)tp.tok_alloc);
    tp.grp_seg = b.take_n<int32_t>((size_t)(tp.tok_alloc / kGroupMin));       // sized for either group size
    tp.chunk_seg = b.take_n<int32_t>((size_t)chunks_alloc);
    return b.ok;
}

hipError_t launch_token_plan(const TokenPlan& tp, const int64_t* row_ptr_batch, const int32_t* col_idx,
                             const float* normE, hipStream_t s)
{
    k_seg_offsets<<<1, kScanThreads, 0, s>>>(row_ptr_batch, tp.nseg, tp.pofs, tp.group);
    int64_t ngroups = tp.tok_alloc / tp.group;
    k_fill_tokens<<<grid_for(ngroups, 256), 256, 0, s>>>(row_ptr_batch, col_idx, (int32_t)tp.nseg, tp.pofs, normE,
                                                         tp.tok_ids, tp.tok_hn, tp.grp_seg, ngroups, tp.group);
    k_chunk_bounds<<<grid_for(tp.nchunks + 1, 256), 256, 0, s>>>(tp.pofs, (int32_t)tp.nseg, tp.chunk_tokens,
                                                                 tp.nchunks, tp.chunk_seg);
    return hipGetLastError();
}

hipError_t launch_zero_matches(const int64_t* row_ptr_batch, const int32_t* col_idx, int64_t nseg,
                               const int32_t* map, float* Z, int64_t ldz, hipStream_t s, uint64_t* bits, int64_t pitch,
                               int slice_words)
{
    if (nseg <= 0) return hipSuccess;
    k_zero_matches<<<(unsigned)((nseg + 3) / 4), 256, 0, s>>>(row_ptr_batch, col_idx, nseg, map, Z, ldz, bits, pitch,
                                                              slice_words > 0 ? slice_words : 64);
    return hipGetLastError();
}

hipError_t launch_redo_close(const void* E, bool bf16, int64_t ld, int32_t m, const float* normE, const int32_t* voc_rows,
                             int64_t nvoc, const int64_t* row_ptr_batch, const int32_t* col_idx, int64_t nseg, float* Z,
                             int64_t ldz, hipStream_t s)
{
    if (nvoc <= 0 || nseg <= 0) return hipSuccess;
    const int64_t strips = (nseg + kRedoCols - 1) / kRedoCols;
    const int64_t grid = (nvoc * strips + 3) / 4;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool vec = (ldz % 4 == 0) && (((uintptr_t)Z & 15) == 0);
#define REDO(B, V) k_redo_close<B, V><<<(unsigned)grid, 256, 0, s>>>(E, ld, m, normE, voc_rows, nvoc, row_ptr_batch, col_idx, nseg, Z, ldz, strips)
    if (bf16) { if (vec) REDO(true, true); else REDO(true, false); }
    else { if (vec) REDO(false, true); else REDO(false, false); }
#undef REDO
    return hipGetLastError();
}

hipError_t launch_redo_close_bits(const void* E, bool bf16, int64_t ld, int32_t m, const int32_t* voc_rows, int64_t nvoc,
                                  const int64_t* row_ptr_batch, const int32_t* col_idx, int64_t nseg, float* Z, int64_t ldz,
                                  const uint64_t* bits, int64_t pitch, int slice_words, hipStream_t s)
{
    if (nvoc <= 0 || nseg <= 0) return hipSuccess;
    const int64_t words = nseg * pitch;
    const int64_t grid = (words + 255) / 256;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    if (bf16) k_redo_close_bits<true><<<(unsigned)grid, 256, 0, s>>>(E, ld, m, voc_rows, nvoc, row_ptr_batch, col_idx, nseg, Z, ldz, bits, pitch, slice_words);
    else k_redo_close_bits<false><<<(unsigned)grid, 256, 0, s>>>(E, ld, m, voc_rows, nvoc, row_ptr_batch, col_idx, nseg, Z, ldz, bits, pitch, slice_words);
    return hipGetLastError();
}

hipError_t launch_validate_csr(const lcrwmd_csr& X, int32_t* status, hipStream_t s)
{
    k_validate_csr<<<grid_for(X.rows > 0 ? X.rows : 1, 256), 256, 0, s>>>(X.row_ptr, X.col_idx, X.val, X.rows,
                                                                          X.cols, X.nnz, status);
    return hipGetLastError();
}

}  // namespace lcrwmd
