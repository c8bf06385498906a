// De-duplicated form of LC-RWMD (Sec. III-IV).  Every histogram entry is a word of the vocabulary, so the Euclidean
// distances the first phase needs are all entries of one word-pair table
//     W[p][u] = || E[db word p] - E[query word u] ||,   p over the distinct database words, u over the distinct
//                                                       words of the query batch,
// which is the operator "o" of Sec. III applied once to the two reduced vocabularies instead of once per stored
// entry.  (Sec. III-B dismisses the full v x v table for its size; the slice belonging to one query batch is small.)
// Both passes then read the table instead of recomputing distances:
//   forward   Z[p][j]  = min_{a in query j} W[p][u_a]                    (k_table_fwd;  D1 = X1 * Z follows as usual)
//   swapped   Z'[u][i] = min_{p in database row i} W[p][u],  D[i][j] = max(D[i][j], sum_a y_ja Z'[u_a][i])
//                                                                         (k_table_rev: both steps fused, Z' stays in LDS)
// The swapped pass is a stream of table rows: 4 * (stored database entries) * (query words) bytes, bandwidth bound.
#include "lcrwmd_internal.h"

namespace lcrwmd {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 1024;            // 16 wavefronts: one workgroup per CU
constexpr int kWaves = kThreads / 64;
constexpr int kSlabMax = 32768;           // floats of a table row held in LDS at a time (128 KiB)

// Identical words are at distance exactly 0; the norm expansion only gets there up to cancellation error.
__global__ void k_table_zero_same(const int32_t* __restrict__ list_q, int32_t vq, const int32_t* __restrict__ map_db,
                                  float* __restrict__ W, int64_t ldw)
{
    const int32_t u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= vq) return;
    const int32_t p = map_db[list_q[u]];
    if (p >= 0) W[(int64_t)p * ldw + u] = 0.f;
}

// Token list of the table launch: the distinct database words, padded with the last one.
__global__ void k_table_tokens(const int32_t* __restrict__ list_db, int32_t ve, const float* __restrict__ normE,
                               int32_t* __restrict__ tok_ids, float* __restrict__ tok_hn, int32_t count)
{
    const int32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= count) return;
    const int32_t id = list_db[t < ve ? t : ve - 1];
    tok_ids[t] = id;
    tok_hn[t] = -0.5f * normE[id];
}

__device__ inline float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}
__device__ inline float wave_min(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fminf(x, __shfl_xor(x, o));
    return x;
}

// Swapped pass, one workgroup per database row i.  The query words are cut into slabs of `slab` (a multiple of 4, at
// most R * 4096) columns.  Per slab: (A) every thread keeps R float4 running minima over the table rows of the
// words of row i (each table row is read as one contiguous, fully coalesced stream); the minima go to LDS; (B) one
// wavefront per query sums weight * minimum over the query's words that fall into the slab.  At the end
// D[i][j] = max(D[i][j], sum_j).  LDS: slab floats + q floats.
template <int R>
__global__ __launch_bounds__(kThreads) void k_table_rev(const float* __restrict__ W, int64_t ldw, int32_t vq,
                                                        int32_t slab, const int64_t* __restrict__ db_rp,
                                                        const int32_t* __restrict__ db_pos,
                                                        const int64_t* __restrict__ q_rp,
                                                        const int32_t* __restrict__ q_pos,
                                                        const float* __restrict__ q_val, int32_t q,
                                                        float* __restrict__ D, int64_t ldd)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float* zrow = lds;             // [slab]
    float* sums = lds + slab;      // [q]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t i = blockIdx.x;
    const int64_t a = db_rp[i], b = db_rp[i + 1];

    for (int j = tid; j < q; j += kThreads) sums[j] = 0.f;

    for (int32_t u0 = 0; u0 < vq; u0 += slab) {
        const int32_t width = vq - u0 < slab ? vq - u0 : slab;     // real columns; the row pitch covers the next multiple of 4
        const int32_t npiece = (width + 3) >> 2;
        // ---- (A) column minima over the row's words ----
        f32x4 best[R];
        bool own[R];
        const float* col[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int k = tid + r * kThreads;
            own[r] = k < npiece;
            col[r] = W + u0 + 4 * (own[r] ? k : 0);
            best[r] = f32x4{INFINITY, INFINITY, INFINITY, INFINITY};
        }
        int64_t p = a;
        for (; p + 1 < b; p += 2) {
            const int64_t o0 = (int64_t)db_pos[p] * ldw, o1 = (int64_t)db_pos[p + 1] * ldw;
            f32x4 x0[R], x1[R];
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (own[r]) {
                    x0[r] = *reinterpret_cast<const f32x4*>(col[r] + o0);
                    x1[r] = *reinterpret_cast<const f32x4*>(col[r] + o1);
                }
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (own[r]) {
#pragma unroll
                    for (int t = 0; t < 4; ++t) best[r][t] = fminf(best[r][t], fminf(x0[r][t], x1[r][t]));
                }
        }
        if (p < b) {
            const int64_t o0 = (int64_t)db_pos[p] * ldw;
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (own[r]) {
                    const f32x4 x = *reinterpret_cast<const f32x4*>(col[r] + o0);
#pragma unroll
                    for (int t = 0; t < 4; ++t) best[r][t] = fminf(best[r][t], x[t]);
                }
        }
        __syncthreads();          // the previous slab's minima are no longer being read
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (own[r]) *reinterpret_cast<f32x4*>(zrow + 4 * (tid + r * kThreads)) = best[r];
        __syncthreads();
        // ---- (B) weighted sums of the queries over this slab ----
        for (int j = wave; j < q; j += kWaves) {
            const int64_t qa = q_rp[j], qb = q_rp[j + 1];
            float part = 0.f;
            for (int64_t e = qa + lane; e < qb; e += 64) {
                const uint32_t c = (uint32_t)(q_pos[e] - u0);
                if (c < (uint32_t)width) part = fmaf(q_val[e], zrow[c], part);
            }
            part = wave_sum(part);
            if (lane == 0) sums[j] += part;       // query j always belongs to this wavefront
        }
    }
    __syncthreads();
    float* drow = D + i * ldd;
    for (int j = tid; j < q; j += kThreads) drow[j] = fmaxf(drow[j], sums[j]);
}

// Forward pass, one workgroup per distinct database word p: the table row goes to LDS slab by slab and one
// wavefront per query takes the minimum over the query's words; Z[p][j] is written once, along the row.
__global__ __launch_bounds__(kThreads) void k_table_fwd(const float* __restrict__ W, int64_t ldw, int32_t vq,
                                                        int32_t slab, const int64_t* __restrict__ q_rp,
                                                        const int32_t* __restrict__ q_pos, int32_t q,
                                                        float* __restrict__ Z, int64_t ldz)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float* wrow = lds;             // [slab]
    float* mins = lds + slab;      // [q]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t p = blockIdx.x;
    const float* row = W + p * ldw;

    for (int j = tid; j < q; j += kThreads) mins[j] = INFINITY;

    for (int32_t u0 = 0; u0 < vq; u0 += slab) {
        const int32_t width = vq - u0 < slab ? vq - u0 : slab;
        const int32_t npiece = (width + 3) >> 2;
        __syncthreads();
        for (int k = tid; k < npiece; k += kThreads)
            *reinterpret_cast<f32x4*>(wrow + 4 * k) = *reinterpret_cast<const f32x4*>(row + u0 + 4 * k);
        __syncthreads();
        for (int j = wave; j < q; j += kWaves) {
            const int64_t qa = q_rp[j], qb = q_rp[j + 1];
            float part = INFINITY;
            for (int64_t e = qa + lane; e < qb; e += 64) {
                const uint32_t c = (uint32_t)(q_pos[e] - u0);
                if (c < (uint32_t)width) part = fminf(part, wrow[c]);
            }
            part = wave_min(part);
            if (lane == 0) mins[j] = fminf(mins[j], part);
        }
    }
    __syncthreads();
    float* zrow = Z + p * ldz;
    for (int j = tid; j < q; j += kThreads) zrow[j] = mins[j];
}

// Slab width for vq columns: the fewest slabs that fit, of equal width (a multiple of 4).
int32_t slab_for(int64_t vq)
{
    const int64_t nslab = (vq + kSlabMax - 1) / kSlabMax;
    int64_t w = (vq + nslab - 1) / nslab;
    w = (w + 3) & ~(int64_t)3;
    return (int32_t)w;
}

}  // namespace

int64_t table_max_queries() { return (160 * 1024 / 4) - kSlabMax; }   // q floats beside a full slab in 160 KiB of LDS

hipError_t launch_table_tokens(const int32_t* list_db, int64_t ve, const float* normE, int32_t* tok_ids, float* tok_hn,
                               int64_t count, hipStream_t s)
{
    if (count <= 0 || ve <= 0) return hipSuccess;
    k_table_tokens<<<(unsigned)((count + 255) / 256), 256, 0, s>>>(list_db, (int32_t)ve, normE, tok_ids, tok_hn, (int32_t)count);
    return hipGetLastError();
}

hipError_t launch_table_zero_same(const int32_t* list_q, int64_t vq, const int32_t* map_db, float* W, int64_t ldw,
                                  hipStream_t s)
{
    if (vq <= 0) return hipSuccess;
    k_table_zero_same<<<(unsigned)((vq + 255) / 256), 256, 0, s>>>(list_q, (int32_t)vq, map_db, W, ldw);
    return hipGetLastError();
}

hipError_t launch_table_fwd(const float* W, int64_t ldw, int64_t ve, int64_t vq, const int64_t* q_rp, const int32_t* q_pos,
                            int64_t q, float* Z, int64_t ldz, hipStream_t s)
{
    if (ve <= 0 || q <= 0 || vq <= 0) return hipSuccess;
    if (q > table_max_queries() || ve > 0x7fffffffLL) return hipErrorInvalidValue;
    const int32_t slab = slab_for(vq);
    const size_t smem = ((size_t)slab + (size_t)q) * 4;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_table_fwd), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    k_table_fwd<<<(unsigned)ve, kThreads, smem, s>>>(W, ldw, (int32_t)vq, slab, q_rp, q_pos, (int32_t)q, Z, ldz);
    return hipGetLastError();
}

template <int R>
static hipError_t launch_rev_r(const float* W, int64_t ldw, int32_t vq, int32_t slab, const int64_t* db_rp,
                               const int32_t* db_pos, int64_t rows, const int64_t* q_rp, const int32_t* q_pos,
                               const float* q_val, int32_t q, float* D, int64_t ldd, size_t smem, hipStream_t s)
{
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_table_rev<R>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    k_table_rev<R><<<(unsigned)rows, kThreads, smem, s>>>(W, ldw, vq, slab, db_rp, db_pos, q_rp, q_pos, q_val, q, D, ldd);
    return hipGetLastError();
}

// D[i][j] = max(D[i][j], sum_a q_val[a] * min_{p in row i} W[db_pos[p]][q_pos[a]]) for i in [0, rows), j in [0, q).
// db_rp is indexed from the first row of the batch and holds offsets into db_pos; the same for q_rp / q_pos / q_val.
hipError_t launch_table_rev(const float* W, int64_t ldw, int64_t vq, const int64_t* db_rp, const int32_t* db_pos,
                            int64_t rows, const int64_t* q_rp, const int32_t* q_pos, const float* q_val, int64_t q,
                            float* D, int64_t ldd, hipStream_t s)
{
    if (rows <= 0 || q <= 0 || vq <= 0) return hipSuccess;
    if (q > table_max_queries() || rows > 0x7fffffffLL || (ldw & 3) != 0 || ((uintptr_t)W & 15) != 0) return hipErrorInvalidValue;
    const int32_t slab = slab_for(vq);
    const size_t smem = ((size_t)slab + (size_t)q) * 4;
    const int r = (slab / 4 + kThreads - 1) / kThreads;
#define REV(RR) return launch_rev_r<RR>(W, ldw, (int32_t)vq, slab, db_rp, db_pos, rows, q_rp, q_pos, q_val, (int32_t)q, D, ldd, smem, s)
    switch (r) {
        case 1: REV(1);
        case 2: REV(2);
        case 3: REV(3);
        case 4: REV(4);
        case 5: REV(5);
        case 6: REV(6);
        case 7: REV(7);
        default: REV(8);
    }
#undef REV
}

}  // namespace lcrwmd
