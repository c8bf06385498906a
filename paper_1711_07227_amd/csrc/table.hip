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
//
// Strips.  The columns u are cut into strips of at most 512 (2 KiB per table row) and the queries' entries are
// regrouped by strip once per call (k_bucket_*).  The swapped pass is launched strip by strip: while one strip is
// being worked on, the strip of the frequent database words' rows stays in the L2s and the strip of the whole table
// fits the Infinity Cache, so most of the stream never reaches HBM; per-strip partial sums accumulate in a buffer
// D2 (always in strip order: the result does not depend on timing).  One wavefront owns one database row: its
// minima live in a private 2 KiB of LDS and no workgroup barrier is needed.
#include "lcrwmd_internal.h"

namespace lcrwmd {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kStrip = 512;               // columns per strip: 2 float4 per lane (measured best of 256 .. 1024 on Medium)
constexpr int kPieces = (kStrip + 255) / 256;     // float4 per lane and table row
constexpr int kWaves = 4;                 // wavefronts per workgroup, each on its own row(s)
constexpr int kMaxQueries = 4096;         // queries per pass: at most 64 per lane in the forward kernel

// Identical words are at distance exactly 0; the norm expansion only gets there up to cancellation error.
__global__ void k_table_zero_same(const int32_t* __restrict__ list_q, int32_t vq, const int32_t* __restrict__ map_db,
                                  float* __restrict__ W, int64_t ldw)
{
    const int32_t u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= vq) return;
    const int32_t p = map_db[list_q[u]];
    if (p >= 0) W[(int64_t)p * ldw + u] = 0.f;
}

// Entries of the table below half the row word's norm (w^2 < |x|^2 / 4) come from a squared distance that is a small
// difference of large numbers in the norm expansion: they are recomputed from coordinate differences, whose error is
// relative to the distance itself.  One wavefront per table row and strip of 1,024 columns; the flagged entries of
// each 64 are redone one after the other, lanes along the embedding dimension.  Equal words (already exactly 0) are
// left alone.  Without close word pairs this is one read of the table.
template <bool BF16>
__global__ __launch_bounds__(256) void k_table_redo_close(const void* __restrict__ E, int64_t ld, int32_t m,
                                                          const float* __restrict__ normE,
                                                          const int32_t* __restrict__ list_db, int64_t ve,
                                                          const int32_t* __restrict__ col_word, int64_t vc,
                                                          float* __restrict__ W, int64_t ldw, int64_t strips)
{
    const int lane = threadIdx.x & 63;
    const int64_t unit = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t p = unit / strips;
    if (p >= ve) return;
    const int64_t strip = unit - p * strips;
    const int32_t w = list_db[p];
    const float limit = 0.25f * normE[w];
    float* row = W + p * ldw;
    // element e of this lane: column c0 + 256 * (e / 4) + 4 * lane + e % 4; table rows are 16-byte aligned and the
    // number of columns is a multiple of 32, so a float4 is inside the row or wholly beyond it
    const int64_t c0 = strip * 1024;
    f32x4 x[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int64_t c = c0 + 256 * b + 4 * lane;
        x[b] = c < vc ? *reinterpret_cast<const f32x4*>(row + c) : f32x4{1e30f, 1e30f, 1e30f, 1e30f};
    }
    bool any = false;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int t = 0; t < 4; ++t) any |= x[b][t] * x[b][t] < limit;
    if (!__any(any)) return;

#pragma unroll 1
    for (int e = 0; e < 16; ++e) {
        const int64_t c = c0 + 256 * (e >> 2) + 4 * lane + (e & 3);
        float xe = x[0][0];
#pragma unroll
        for (int t = 1; t < 16; ++t) xe = e == t ? x[t >> 2][t & 3] : xe;
        const int32_t cw = c < vc ? col_word[c] : w;
        uint64_t todo = __ballot(xe * xe < limit && cw != w);
        while (todo) {
            const int l = __builtin_ctzll(todo);
            todo &= todo - 1;
            const int32_t u = __builtin_amdgcn_readlane(cw, l);
            float sum = 0.f;
            for (int32_t k = lane; k < m; k += 64) {
                float a, b;
                if (BF16) {
                    a = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(E)[(int64_t)w * ld + k] << 16);
                    b = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(E)[(int64_t)u * ld + k] << 16);
                } else {
                    a = reinterpret_cast<const float*>(E)[(int64_t)w * ld + k];
                    b = reinterpret_cast<const float*>(E)[(int64_t)u * ld + k];
                }
                sum = fmaf(a - b, a - b, sum);
            }
            for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
            if (lane == l) row[c] = sqrtf(sum);
        }
    }
}

// Columns of the table: query word number u (in increasing word id) goes to strip u mod nstrip, place u / nstrip.
// Word ids grow with rarity in real vocabularies, so this deals the frequent words out over all strips: every
// strip then sees about the same number of entries per query (with the words in id order the first strip held
// nearly all of them and its per-query loops dominated).  Unused places at the end of a strip repeat word 0 of
// the list; no entry points at them.
__global__ void k_spread_columns(const int32_t* __restrict__ list_q, int32_t vq, int32_t ws, int32_t nstrip,
                                 int32_t* __restrict__ col_word)
{
    const int32_t c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= ws * nstrip) return;
    const int32_t u = (c % ws) * nstrip + c / ws;
    col_word[c] = list_q[u < vq ? u : 0];
}

__global__ void k_spread_entries(const int32_t* __restrict__ pos_in, int64_t nnz, int32_t ws, int32_t nstrip,
                                 int32_t* __restrict__ pos_out)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= nnz) return;
    const int32_t u = pos_in[e];
    pos_out[e] = (u % nstrip) * ws + u / nstrip;
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

// ---- the queries' entries regrouped by strip ----
// offs[s * q + j] = start of the entries of query j that fall into strip s, in (strip, query) order; offs[nstrip * q]
// = their number.  bpos = column - strip start, bval = weight; the entries of one (strip, query) keep their order.

// One thread per query: counts per strip.
__global__ void k_bucket_count(const int64_t* __restrict__ q_rp, const int32_t* __restrict__ q_pos, int32_t q,
                               int32_t ws, int32_t nstrip, int32_t* __restrict__ cnt)
{
    const int32_t j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= q) return;
    for (int32_t s = 0; s < nstrip; ++s) cnt[(int64_t)s * q + j] = 0;
    for (int64_t e = q_rp[j]; e < q_rp[j + 1]; ++e) cnt[(int64_t)(q_pos[e] / ws) * q + j] += 1;
}

// Single workgroup: offs = exclusive prefix sums of cnt[0 .. count), offs[count] = total; cursor = copy of offs.
__global__ __launch_bounds__(1024) void k_bucket_scan(const int32_t* __restrict__ cnt, int64_t count,
                                                      int32_t* __restrict__ offs, int32_t* __restrict__ cursor)
{
    __shared__ int32_t wsum[17];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t carry = 0;
    for (int64_t base = 0; base < count; base += 1024) {
        const int64_t k = base + threadIdx.x;
        const int32_t x = k < count ? cnt[k] : 0;
        int32_t incl = x;
        for (int o = 1; o < 64; o <<= 1) {
            const int32_t y = __shfl_up(incl, o);
            if (lane >= o) incl += y;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        if (threadIdx.x == 0) {
            int32_t run = 0;
            for (int w = 0; w < 16; ++w) { const int32_t t = wsum[w]; wsum[w] = run; run += t; }
            wsum[16] = run;
        }
        __syncthreads();
        const int32_t excl = carry + wsum[wave] + incl - x;
        if (k < count) { offs[k] = excl; cursor[k] = excl; }
        carry += wsum[16];
        __syncthreads();
    }
    if (threadIdx.x == 0) offs[count] = carry;
}

// One thread per query: entries to their places.  cursor[s * q + j] is private to the thread.
__global__ void k_bucket_scatter(const int64_t* __restrict__ q_rp, const int32_t* __restrict__ q_pos,
                                 const float* __restrict__ q_val, int32_t q, int32_t ws, int32_t* __restrict__ cursor,
                                 int32_t* __restrict__ bpos, float* __restrict__ bval)
{
    const int32_t j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= q) return;
    int32_t cur_s = -1, cur = 0;
    for (int64_t e = q_rp[j]; e < q_rp[j + 1]; ++e) {
        const int32_t c = q_pos[e], s = c / ws;
        if (s != cur_s) {
            if (cur_s >= 0) cursor[(int64_t)cur_s * q + j] = cur;
            cur_s = s;
            cur = cursor[(int64_t)s * q + j];
        }
        bpos[cur] = c - s * ws;
        bval[cur] = q_val[e];
        ++cur;
    }
}

// Make this wavefront's LDS writes visible to its own later reads (one wavefront = one owner of the region).
__device__ inline void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Swapped pass over one strip [c0, c0 + 4 * npiece) of the columns; one wavefront per database row i.
//   (A) lanes keep float4 running minima over the table rows of the words of row i (each row segment is read as
//       one contiguous piece), then park them in LDS;
//   (B) lane = query: sum of weight * minimum over the query's entries in this strip, added to the partial sum of
//       the strips before (D2); the last strip applies the maximum with D instead.
__global__ __launch_bounds__(64 * kWaves) void k_table_rev(const float* __restrict__ W, int64_t ldw, int32_t c0,
                                                          int32_t npiece, const int64_t* __restrict__ db_rp,
                                                          const int32_t* __restrict__ db_pos, int64_t n,
                                                          const int32_t* __restrict__ brp,
                                                          const int32_t* __restrict__ bpos,
                                                          const float* __restrict__ bval, int32_t q,
                                                          float* __restrict__ D2, int64_t ld2, float* __restrict__ D,
                                                          int64_t ldd, int first, int last)
{
    __shared__ __attribute__((aligned(16))) float zs[kWaves][kStrip];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t i = (int64_t)blockIdx.x * kWaves + wave;
    if (i >= n) return;                       // whole wavefronts leave; there is no workgroup barrier below
    const int64_t a = db_rp[i], b = db_rp[i + 1];

    const float* col[kPieces];
    f32x4 best[kPieces];
#pragma unroll
    for (int r = 0; r < kPieces; ++r) {
        const int piece = lane + 64 * r;
        col[r] = W + c0 + 4 * (piece < npiece ? piece : 0);      // lanes without a piece re-read piece 0
        best[r] = f32x4{INFINITY, INFINITY, INFINITY, INFINITY};
    }
    int64_t p = a;
    constexpr int UN = 4;                       // table rows in flight per lane and piece (8 measured slower)
    for (; p + UN - 1 < b; p += UN) {
        int64_t o[UN];
#pragma unroll
        for (int t = 0; t < UN; ++t) o[t] = (int64_t)db_pos[p + t] * ldw;
        f32x4 x[UN][kPieces];
#pragma unroll
        for (int t = 0; t < UN; ++t)
#pragma unroll
            for (int r = 0; r < kPieces; ++r) x[t][r] = *reinterpret_cast<const f32x4*>(col[r] + o[t]);
#pragma unroll
        for (int r = 0; r < kPieces; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float m = best[r][c];
#pragma unroll
                for (int t = 0; t < UN; ++t) m = fminf(m, x[t][r][c]);
                best[r][c] = m;
            }
    }
    for (; p < b; ++p) {
        const int64_t o = (int64_t)db_pos[p] * ldw;
#pragma unroll
        for (int r = 0; r < kPieces; ++r) {
            const f32x4 x = *reinterpret_cast<const f32x4*>(col[r] + o);
#pragma unroll
            for (int c = 0; c < 4; ++c) best[r][c] = fminf(best[r][c], x[c]);
        }
    }
#pragma unroll
    for (int r = 0; r < kPieces; ++r)
        if (lane + 64 * r < npiece) *reinterpret_cast<f32x4*>(&zs[wave][4 * (lane + 64 * r)]) = best[r];
    wave_lds_sync();

    const float* z = zs[wave];
    float* d2 = D2 + i * ld2;
    float* d = D + i * ldd;
    // Eight slices of 64 queries at a time: their entry ranges, the partial sums so far and the values of D are all
    // requested before the first is used, and the first four entries of every slice are in flight together.
    constexpr int SL = 8;
    for (int32_t jb = 0; jb < q; jb += 64 * SL) {
        int32_t ea[SL], eb[SL];
        float prev[SL], dold[SL];
#pragma unroll
        for (int k = 0; k < SL; ++k) {
            const int32_t j = jb + 64 * k + lane;
            const bool ok = j < q;
            ea[k] = ok ? brp[j] : 0;
            eb[k] = ok ? brp[j + 1] : 0;
            prev[k] = (ok && !first) ? d2[j] : 0.f;
            dold[k] = (ok && last) ? d[j] : 0.f;
        }
        int32_t c[SL][4];
        float w[SL][4];
#pragma unroll
        for (int k = 0; k < SL; ++k)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const bool ok = ea[k] + t < eb[k];
                c[k][t] = ok ? bpos[ea[k] + t] : 0;
                w[k][t] = ok ? bval[ea[k] + t] : 0.f;
            }
#pragma unroll
        for (int k = 0; k < SL; ++k) {
            const int32_t j = jb + 64 * k + lane;
            float acc = 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t) acc = fmaf(w[k][t], z[c[k][t]], acc);      // entry order, as in the loop below
            for (int32_t e = ea[k] + 4; e < eb[k]; e += 4) {
                int32_t cc[4];
                float ww[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const bool ok = e + t < eb[k];
                    cc[t] = bpos[ok ? e + t : e];
                    ww[t] = ok ? bval[e + t] : 0.f;
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) acc = fmaf(ww[t], z[cc[t]], acc);
            }
            acc += prev[k];
            if (j < q) {
                if (last) d[j] = fmaxf(dold[k], acc);
                else d2[j] = acc;
            }
        }
    }
}

// Forward pass: one wavefront per RW table rows, all strips in turn.  Lane l owns the queries l, l + 64, ...
// (QPL of them) and keeps their running minima for the RW rows in registers; a strip of the RW rows is parked in
// LDS, then every owned query walks its entries of that strip.  Z[p][j] is written once, along the row.
template <int QPL, int RW>
__global__ __launch_bounds__(64 * kWaves) void k_table_fwd(const float* __restrict__ W, int64_t ldw, int64_t ve,
                                                          int32_t vq, int32_t ws, int32_t nstrip,
                                                          const int32_t* __restrict__ offs,
                                                          const int32_t* __restrict__ bpos, int32_t q,
                                                          float* __restrict__ Z, int64_t ldz)
{
    __shared__ __attribute__((aligned(16))) float zs[kWaves][RW][kStrip];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t p0 = ((int64_t)blockIdx.x * kWaves + wave) * RW;
    if (p0 >= ve) return;
    const float* row[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) row[r] = W + (p0 + r < ve ? p0 + r : ve - 1) * ldw;
    float acc[RW][QPL];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int jj = 0; jj < QPL; ++jj) acc[r][jj] = INFINITY;

    for (int32_t s = 0; s < nstrip; ++s) {
        const int32_t c0 = s * ws;
        const int32_t width = vq - c0 < ws ? vq - c0 : ws;
        const int32_t npiece = (width + 3) >> 2;
        wave_lds_sync();                       // the previous strip has been read
#pragma unroll
        for (int r = 0; r < RW; ++r)
#pragma unroll
            for (int k = 0; k < kPieces; ++k) {
                const int piece = lane + 64 * k;
                if (piece < npiece)
                    *reinterpret_cast<f32x4*>(&zs[wave][r][4 * piece]) = *reinterpret_cast<const f32x4*>(row[r] + c0 + 4 * piece);
            }
        wave_lds_sync();
        const int32_t* brp = offs + (int64_t)s * q;
#pragma unroll
        for (int jj = 0; jj < QPL; ++jj) {
            const int32_t j = lane + 64 * jj;
            if (j < q) {
                const int32_t ea = brp[j], eb = brp[j + 1];
                for (int32_t e = ea; e < eb; e += 4) {      // four entries' loads in flight; a repeated entry changes no minimum
                    int32_t c[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) c[t] = bpos[e + t < eb ? e + t : e];
#pragma unroll
                    for (int r = 0; r < RW; ++r)
                        acc[r][jj] = fminf(fminf(acc[r][jj], fminf(zs[wave][r][c[0]], zs[wave][r][c[1]])),
                                           fminf(zs[wave][r][c[2]], zs[wave][r][c[3]]));
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RW; ++r)
        if (p0 + r < ve) {
            float* zrow = Z + (p0 + r) * ldz;
#pragma unroll
            for (int jj = 0; jj < QPL; ++jj)
                if (lane + 64 * jj < q) zrow[lane + 64 * jj] = acc[r][jj];
        }
}

}  // namespace

int64_t table_max_queries() { return kMaxQueries; }

// Strips for vq columns: equal widths, multiples of 32, at most kStrip.
void table_strips(int64_t vq, int32_t* ws, int32_t* nstrip)
{
    const int64_t ns = vq > 0 ? (vq + kStrip - 1) / kStrip : 1;
    int64_t w = (vq + ns - 1) / ns;
    w = (w + 31) & ~(int64_t)31;            // strips start on 128-byte lines of the table rows
    if (w < 32) w = 32;
    *ws = (int32_t)w;
    *nstrip = (int32_t)((vq + w - 1) / w > 0 ? (vq + w - 1) / w : 1);
}

// Bytes of the regrouped query entries (offs, cursor / counts, bpos, bval) for q queries with nnz_q entries.
size_t table_bucket_bytes(int64_t vq, int64_t q, int64_t nnz_q)
{
    int32_t ws, ns;
    table_strips(vq, &ws, &ns);
    return 3 * (((size_t)ns * (size_t)q + 1) * 4 + 256) + 3 * ((size_t)nnz_q * 4 + 256) + (size_t)ws * ns * 4 + 256;
}

// Deal the vq query words out over the strips: col_word[ws * nstrip] = word of every table column, pos_out = the
// entries' columns (pos_in holds their numbers in the word list).
hipError_t launch_table_spread(const int32_t* list_q, int64_t vq, const int32_t* pos_in, int64_t nnz, int32_t* col_word,
                               int32_t* pos_out, hipStream_t s)
{
    if (vq <= 0) return hipSuccess;
    int32_t ws, ns;
    table_strips(vq, &ws, &ns);
    const int64_t cols = (int64_t)ws * ns;
    k_spread_columns<<<(unsigned)((cols + 255) / 256), 256, 0, s>>>(list_q, (int32_t)vq, ws, ns, col_word);
    if (nnz > 0) k_spread_entries<<<(unsigned)((nnz + 255) / 256), 256, 0, s>>>(pos_in, nnz, ws, ns, pos_out);
    return hipGetLastError();
}

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

hipError_t launch_table_redo_close(const void* E, bool bf16, int64_t ld, int32_t m, const float* normE,
                                   const int32_t* list_db, int64_t ve, const int32_t* col_word, int64_t vc, float* W,
                                   int64_t ldw, hipStream_t s)
{
    if (ve <= 0 || vc <= 0) return hipSuccess;
    const int64_t strips = (vc + 1023) / 1024;
    const int64_t grid = (ve * strips + 3) / 4;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    if (bf16) k_table_redo_close<true><<<(unsigned)grid, 256, 0, s>>>(E, ld, m, normE, list_db, ve, col_word, vc, W, ldw, strips);
    else k_table_redo_close<false><<<(unsigned)grid, 256, 0, s>>>(E, ld, m, normE, list_db, ve, col_word, vc, W, ldw, strips);
    return hipGetLastError();
}

// Regroup the entries of q queries (q_rp indexed from the first query of the batch, offsets into q_pos / q_val).
// cnt, offs and cursor hold nstrip * q + 1 values each.
hipError_t launch_table_buckets(const int64_t* q_rp, const int32_t* q_pos, const float* q_val, int64_t q, int64_t vq,
                                int32_t* cnt, int32_t* offs, int32_t* cursor, int32_t* bpos, float* bval, hipStream_t s)
{
    if (q <= 0) return hipSuccess;
    int32_t ws, ns;
    table_strips(vq, &ws, &ns);
    const unsigned grid = (unsigned)((q + 63) / 64);
    k_bucket_count<<<grid, 64, 0, s>>>(q_rp, q_pos, (int32_t)q, ws, ns, cnt);
    k_bucket_scan<<<1, 1024, 0, s>>>(cnt, (int64_t)ns * q, offs, cursor);
    k_bucket_scatter<<<grid, 64, 0, s>>>(q_rp, q_pos, q_val, (int32_t)q, ws, cursor, bpos, bval);
    return hipGetLastError();
}

hipError_t launch_table_fwd(const float* W, int64_t ldw, int64_t ve, int64_t vq, const int32_t* offs, const int32_t* bpos,
                            int64_t q, float* Z, int64_t ldz, hipStream_t s)
{
    if (ve <= 0 || q <= 0 || vq <= 0) return hipSuccess;
    if (q > kMaxQueries || (ldw & 3) != 0 || ((uintptr_t)W & 15) != 0) return hipErrorInvalidValue;
    int32_t ws, ns;
    table_strips(vq, &ws, &ns);
#define FWD(QPL, RW)                                                                                                   \
    do {                                                                                                               \
        const int64_t grid = (ve + (int64_t)kWaves * RW - 1) / ((int64_t)kWaves * RW);                                 \
        if (grid > 0x7fffffffLL) return hipErrorInvalidValue;                                                          \
        k_table_fwd<QPL, RW><<<(unsigned)grid, 64 * kWaves, 0, s>>>(W, ldw, ve, (int32_t)vq, ws, ns, offs, bpos, (int32_t)q, Z, ldz); \
    } while (0)
    if (q <= 4 * 64) FWD(4, 4);
    else if (q <= 16 * 64) FWD(16, 4);
    else if (q <= 32 * 64) FWD(32, 2);
    else FWD(64, 1);
#undef FWD
    return hipGetLastError();
}

// D[i][j] = max(D[i][j], sum_a bval[a] * min_{p in row i} W[db_pos[p]][column of a]) for i in [0, rows), j in [0, q).
// db_rp is indexed from the first row of the batch and holds offsets into db_pos.  D2 (rows x ld2) holds the partial
// sums between the strips' launches.
hipError_t launch_table_rev(const float* W, int64_t ldw, int64_t vq, const int64_t* db_rp, const int32_t* db_pos,
                            int64_t rows, const int32_t* offs, const int32_t* bpos, const float* bval, int64_t q,
                            float* D2, int64_t ld2, float* D, int64_t ldd, hipStream_t s)
{
    if (rows <= 0 || q <= 0 || vq <= 0) return hipSuccess;
    if (q > kMaxQueries || (ldw & 3) != 0 || ((uintptr_t)W & 15) != 0) return hipErrorInvalidValue;
    int32_t ws, ns;
    table_strips(vq, &ws, &ns);
    const int64_t grid = (rows + kWaves - 1) / kWaves;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    for (int32_t st = 0; st < ns; ++st) {
        const int32_t c0 = st * ws;
        const int32_t width = (int32_t)(vq - c0 < ws ? vq - c0 : ws);
        k_table_rev<<<(unsigned)grid, 64 * kWaves, 0, s>>>(W, ldw, c0, (width + 3) >> 2, db_rp, db_pos, rows, offs + (int64_t)st * q,
                                                          bpos, bval, (int32_t)q, D2, ld2, D, ldd, st == 0, st == ns - 1);
    }
    return hipGetLastError();
}

}  // namespace lcrwmd
