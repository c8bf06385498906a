// First phase of LC-RWMD, fp32 (Sec. IV, Fig. 6, many-to-many form): the row-wise minima, taken
// separately per histogram, of E o T where T stacks the word vectors of a batch of histograms.
//
//   Z[w][j] = sqrt(max(|E_w|^2 - 2 * max_{a in seg j} (T_a . E_w - |T_a|^2 / 2), 0))
//
// The T.E^T contraction runs on the matrix cores (v_mfma_f32_32x32x2_f32) with token rows as the
// M dimension and vocabulary words as the N dimension: in the 32x32 accumulator a lane then holds
// ONE vocabulary word and 16 token rows, so the minimum over tokens is lane-local except for one
// exchange between the two lane halves when a histogram ends.  Histograms are padded to groups of
// 8 tokens (lcrwmd_internal.h), so every 4-register group of the accumulator belongs to one
// histogram and the epilogue's control flow is wave-uniform.  The pairwise matrix C of the paper
// only ever exists in accumulators.
//
// Work decomposition: a workgroup owns 128 vocabulary words (4 wavefronts x 32) and one chunk of
// whole histograms; it walks the chunk's token tiles (128 rows) and K in pieces of 60, staging
// both operands through LDS.  Token vectors are gathered straight from E by word id, the stacked
// T matrix is never materialised.
#include "lcrwmd_internal.h"

namespace lcrwmd {

namespace {

constexpr int KC = 60;             // K piece staged in LDS (300 = 5 * 60)
constexpr int KS = 62;             // LDS row pitch in floats: 2*odd keeps 8-byte reads conflict free
constexpr int STEPS = KC / 4;      // each step feeds two 32x32x2 MFMAs per tile
constexpr int SLOTS = kTileTokens / 16;   // rows staged per thread and operand (16 threads share a row)

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct P1Dev {
    const float* E;
    int64_t ld;
    int32_t m;
    int32_t nkc;
    const float* normE;
    const int32_t* voc_rows;
    int64_t nvoc;
    int32_t z_by_position;
    int32_t nvt;
    int32_t nchunks;
    const int32_t* pofs;
    const int32_t* tok_ids;
    const float* tok_hn;
    const int32_t* grp_seg;
    const int32_t* chunk_seg;
    float* Z;
    int64_t ldz;
};

// Four consecutive values of a row starting at column k, zero beyond column m.  Loads are always in
// bounds (the address falls back to the start of the row) and the zeroing is a select, so a run of these
// loads stays one straight-line burst.
template <bool VEC>
__device__ inline float4 load4(const float* row, int k, int m)
{
    if (VEC) {   // m % 4 == 0 and 16-byte aligned rows: k < m implies k + 3 < m
        const bool in = k < m;
        float4 r = *reinterpret_cast<const float4*>(row + (in ? k : 0));
        if (!in) r = make_float4(0.f, 0.f, 0.f, 0.f);
        return r;
    } else {
        float x[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const bool in = k + t < m;
            const float y = row[in ? k + t : 0];
            x[t] = in ? y : 0.f;
        }
        return make_float4(x[0], x[1], x[2], x[3]);
    }
}

template <bool VEC>
__global__ __launch_bounds__(256, 1) void k_phase1_f32_lds(P1Dev p)
{
    __shared__ float As[kTileTokens * KS];   // token rows
    __shared__ float Bs[kTileVocab * KS];    // vocabulary rows

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l31 = lane & 31, half = lane >> 5;

    // Work item -> (chunk, vocabulary tile).  Consecutive workgroup ids land on different XCDs, so
    // each XCD is given a contiguous range of items: its co-resident workgroups share one chunk's
    // token rows through that XCD's L2.
    const int64_t items = (int64_t)p.nvt * p.nchunks;
    const int64_t per_xcd = (items + 7) >> 3;
    const int64_t slot = blockIdx.x >> 3;
    const int64_t item = (int64_t)(blockIdx.x & 7) * per_xcd + slot;
    if (slot >= per_xcd || item >= items) return;
    const int chunk = (int)(item / p.nvt);
    const int vt = (int)(item - (int64_t)chunk * p.nvt);

    const int s0 = p.chunk_seg[chunk], s1 = p.chunk_seg[chunk + 1];
    if (s0 >= s1) return;
    const int t0 = p.pofs[s0], t1 = p.pofs[s1];
    if (t0 >= t1) return;

    // this lane's vocabulary word
    const int64_t col = (int64_t)vt * kTileVocab + wave * 32 + l31;
    const bool col_ok = col < p.nvoc;
    const int64_t colc = col_ok ? col : p.nvoc - 1;
    const int32_t wid = p.voc_rows ? p.voc_rows[colc] : (int32_t)colc;
    const float nEw = p.normE[wid];
    float* zout = p.Z + (p.z_by_position ? colc : (int64_t)wid) * p.ldz;

    // Staging layout: 16 threads per row (15 float4 pieces of a 60-wide K piece, one thread idles), so
    // slot i of a thread is row (tid >> 4) + 16 i of the tile and its K offset is the same in every slot.
    const int lrow = tid >> 4;
    const int lk = (tid & 15) * 4;
    const bool lactive = (tid & 15) < KC / 4;
    int32_t bword[SLOTS], aword[SLOTS];
#pragma unroll
    for (int i = 0; i < SLOTS; ++i) {
        int64_t vc = (int64_t)vt * kTileVocab + lrow + 16 * i;
        if (vc >= p.nvoc) vc = p.nvoc - 1;
        bword[i] = p.voc_rows ? p.voc_rows[vc] : (int32_t)vc;
    }

    float4 pa[SLOTS], pb[SLOTS];

    auto set_tile_rows = [&](int tb) {
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) aword[i] = p.tok_ids[tb + lrow + 16 * i];
    };
    auto prefetch = [&](int kc) {
        const int k = kc * KC + lk;
        if (lactive) {
#pragma unroll
            for (int i = 0; i < SLOTS; ++i) {
                pa[i] = load4<VEC>(p.E + (int64_t)aword[i] * p.ld, k, p.m);
                pb[i] = load4<VEC>(p.E + (int64_t)bword[i] * p.ld, k, p.m);
            }
        }
    };
    auto stage = [&]() {
        if (lactive) {
#pragma unroll
            for (int i = 0; i < SLOTS; ++i) {
                float* da = &As[(lrow + 16 * i) * KS + lk];
                float* db = &Bs[(lrow + 16 * i) * KS + lk];
                *reinterpret_cast<float2*>(da) = make_float2(pa[i].x, pa[i].y);
                *reinterpret_cast<float2*>(da + 2) = make_float2(pa[i].z, pa[i].w);
                *reinterpret_cast<float2*>(db) = make_float2(pb[i].x, pb[i].y);
                *reinterpret_cast<float2*>(db + 2) = make_float2(pb[i].z, pb[i].w);
            }
        }
    };

    f32x16 acc[4];
    int cur = -1;        // histogram whose running maximum is held in `run`
    float run = 0.f;

    auto flush = [&]() {
        if (cur >= 0) {
            float other = __shfl_xor(run, 32);
            float best = fmaxf(run, other);
            if (half == 0 && col_ok) zout[cur] = sqrtf(fmaxf(nEw - 2.f * best, 0.f));
        }
    };

    set_tile_rows(t0);
    prefetch(0);

    for (int tb = t0; tb < t1; tb += kTileTokens) {
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rt][r] = 0.f;

        float hn[4];
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) hn[rt] = half == 0 ? p.tok_hn[tb + rt * 32 + l31] : 0.f;

        for (int kc = 0; kc < p.nkc; ++kc) {
            __syncthreads();          // everyone finished reading the previous piece
            stage();
            __syncthreads();
            // next piece's global loads fly while this piece is multiplied
            if (kc + 1 < p.nkc) {
                prefetch(kc + 1);
            } else if (tb + kTileTokens < t1) {
                set_tile_rows(tb + kTileTokens);
                prefetch(0);
            }
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const float2 b = *reinterpret_cast<const float2*>(&Bs[(wave * 32 + l31) * KS + 4 * s + 2 * half]);
#pragma unroll
                for (int rt = 0; rt < 4; ++rt) {
                    const float2 a =
                        *reinterpret_cast<const float2*>(&As[(rt * 32 + l31) * KS + 4 * s + 2 * half]);
                    acc[rt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc[rt], 0, 0, 0);
                    acc[rt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc[rt], 0, 0, 0);
                }
            }
        }
        // one more rank-1 step adds -|T_a|^2/2 to every element of token row a
        {
            const float one = half == 0 ? 1.f : 0.f;
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) acc[rt] = __builtin_amdgcn_mfma_f32_32x32x2f32(hn[rt], one, acc[rt], 0, 0, 0);
        }
        // Epilogue: accumulator registers 4g..4g+3 of row tile rt hold token rows 32rt+8g+4*half+{0..3}
        // of this lane's vocabulary word, i.e. group 4rt+g of the tile.
        int ng = (t1 - tb) >> 3;
        if (ng > 16) ng = 16;
        const int32_t* gs = p.grp_seg + (tb >> 3);
#pragma unroll
        for (int g = 0; g < 16; ++g) {
            if (g < ng) {
                const int sg = gs[g];
                const int rt = g >> 2, r0 = (g & 3) * 4;
                const float mg = fmaxf(fmaxf(acc[rt][r0], acc[rt][r0 + 1]), fmaxf(acc[rt][r0 + 2], acc[rt][r0 + 3]));
                if (sg != cur) {
                    flush();
                    cur = sg;
                    run = mg;
                } else {
                    run = fmaxf(run, mg);
                }
            }
        }
    }
    flush();
}

// ---------------------------------------------------------------------------------------------------
// Fast path for m <= 300: the vocabulary operand never leaves registers.
//
// A lane's share of its wavefront's 32 vocabulary words is one word x (m / 2) values = at most 150
// VGPRs, loaded once per workgroup.  Only token rows stream through LDS (double buffered, one barrier
// per K piece), which halves LDS and L2 traffic against staging both operands and leaves the L2 to the
// token rows that the workgroups of an XCD share.  One workgroup per CU (512 registers per lane).
// ---------------------------------------------------------------------------------------------------
constexpr int MAXKC = 5;                    // K pieces held in registers: m <= MAXKC * KC = 300

template <bool VEC>
__global__ __launch_bounds__(256, 1) void k_phase1_f32_regb(P1Dev p)
{
    __shared__ float As[2][kTileTokens * KS];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l31 = lane & 31, half = lane >> 5;

    const int64_t items = (int64_t)p.nvt * p.nchunks;
    const int64_t per_xcd = (items + 7) >> 3;
    const int64_t slot = blockIdx.x >> 3;
    const int64_t item = (int64_t)(blockIdx.x & 7) * per_xcd + slot;
    if (slot >= per_xcd || item >= items) return;
    const int chunk = (int)(item / p.nvt);
    const int vt = (int)(item - (int64_t)chunk * p.nvt);

    const int s0 = p.chunk_seg[chunk], s1 = p.chunk_seg[chunk + 1];
    if (s0 >= s1) return;
    const int t0 = p.pofs[s0], t1 = p.pofs[s1];
    if (t0 >= t1) return;

    const int64_t col = (int64_t)vt * kTileVocab + wave * 32 + l31;
    const bool col_ok = col < p.nvoc;
    const int64_t colc = col_ok ? col : p.nvoc - 1;
    const int32_t wid = p.voc_rows ? p.voc_rows[colc] : (int32_t)colc;
    const float nEw = p.normE[wid];
    float* zout = p.Z + (p.z_by_position ? colc : (int64_t)wid) * p.ldz;

    // staging: 16 threads per row, slot i of a thread is row (tid >> 4) + 16 i
    const int lrow = tid >> 4;
    // the 16th thread of a row repeats the 15th piece: same value to the same place, and no divergence
    const int lk = ((tid & 15) < KC / 4 ? (tid & 15) : KC / 4 - 1) * 4;
    float4 pa[SLOTS];
    int32_t aword[SLOTS], aword_next[SLOTS];

    auto stage = [&](float* dst) {
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            float* d = dst + (lrow + 16 * i) * KS + lk;
            *reinterpret_cast<float2*>(d) = make_float2(pa[i].x, pa[i].y);
            *reinterpret_cast<float2*>(d + 2) = make_float2(pa[i].z, pa[i].w);
        }
    };

    // ---- vocabulary operand -> registers (through LDS so that the global reads are contiguous) ----
    float2 breg[MAXKC * STEPS];
    {
        int32_t bword[SLOTS];
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            int64_t vc = (int64_t)vt * kTileVocab + lrow + 16 * i;
            if (vc >= p.nvoc) vc = p.nvoc - 1;
            bword[i] = p.voc_rows ? p.voc_rows[vc] : (int32_t)vc;
        }
#pragma unroll
        for (int kc = 0; kc < MAXKC; ++kc) {
            if (kc < p.nkc) {
#pragma unroll
                for (int i = 0; i < SLOTS; ++i)
                    pa[i] = load4<VEC>(p.E + (int64_t)bword[i] * p.ld, kc * KC + lk, p.m);
                __syncthreads();
                stage(As[0]);
                __syncthreads();
#pragma unroll
                for (int s = 0; s < STEPS; ++s)
                    breg[kc * STEPS + s] =
                        *reinterpret_cast<const float2*>(&As[0][(wave * 32 + l31) * KS + 4 * s + 2 * half]);
            } else {
#pragma unroll
                for (int s = 0; s < STEPS; ++s) breg[kc * STEPS + s] = make_float2(0.f, 0.f);
            }
        }
        __syncthreads();
    }

    auto load_tile_words = [&](int tb, int32_t* w) {
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) w[i] = p.tok_ids[tb + lrow + 16 * i];
    };
    auto prefetch = [&](int kc) {
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) pa[i] = load4<VEC>(p.E + (int64_t)aword[i] * p.ld, kc * KC + lk, p.m);
    };

    f32x16 acc[4];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int cur = -1;
    float run = 0.f;
    auto flush = [&]() {
        if (cur >= 0) {
            float other = __shfl_xor(run, 32);
            float best = fmaxf(run, other);
            if (half == 0 && col_ok) zout[cur] = sqrtf(fmaxf(nEw - 2.f * best, 0.f));
        }
    };

    load_tile_words(t0, aword);
    prefetch(0);
    stage(As[0]);
    __syncthreads();
    int buf = 0;

    for (int tb = t0; tb < t1; tb += kTileTokens) {
        const bool more = tb + kTileTokens < t1;
        if (more) load_tile_words(tb + kTileTokens, aword_next);
        float hn[4];
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) hn[rt] = half == 0 ? p.tok_hn[tb + rt * 32 + l31] : 0.f;
        // histogram of each of the tile's 16 token groups: lane g keeps group g, read back with readlane
        const int gsv = p.grp_seg[(tb >> 3) + (lane & 15)];

#pragma unroll
        for (int kc = 0; kc < MAXKC; ++kc) {
            if (kc < p.nkc) {
                // the next piece's global loads fly while this piece is multiplied
                const bool last = kc + 1 >= p.nkc;
                if (!last) {
                    prefetch(kc + 1);
                } else if (more) {
#pragma unroll
                    for (int i = 0; i < SLOTS; ++i) aword[i] = aword_next[i];
                    prefetch(0);
                }
                const float* A = As[buf] + l31 * KS + 2 * half;
#pragma unroll
                for (int s = 0; s < STEPS; ++s) {
                    float2 a[4];
#pragma unroll
                    for (int rt = 0; rt < 4; ++rt) a[rt] = *reinterpret_cast<const float2*>(A + rt * 32 * KS + 4 * s);
                    const float2 b = breg[kc * STEPS + s];
                    // the first step of a tile starts from a zero accumulator (an inline constant, no clearing pass)
#pragma unroll
                    for (int rt = 0; rt < 4; ++rt)
                        acc[rt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[rt].x, b.x, (kc == 0 && s == 0) ? zero16 : acc[rt], 0, 0, 0);
#pragma unroll
                    for (int rt = 0; rt < 4; ++rt) acc[rt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[rt].y, b.y, acc[rt], 0, 0, 0);
                }
                if (!last || more) stage(As[buf ^ 1]);
                __syncthreads();
                buf ^= 1;
            }
        }
        {
            const float one = half == 0 ? 1.f : 0.f;
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) acc[rt] = __builtin_amdgcn_mfma_f32_32x32x2f32(hn[rt], one, acc[rt], 0, 0, 0);
        }
        int ng = (t1 - tb) >> 3;
        if (ng > 16) ng = 16;
#pragma unroll
        for (int g = 0; g < 16; ++g) {
            if (g < ng) {
                const int sg = __builtin_amdgcn_readlane(gsv, g);
                const int rt = g >> 2, r0 = (g & 3) * 4;
                const float mg = fmaxf(fmaxf(acc[rt][r0], acc[rt][r0 + 1]), fmaxf(acc[rt][r0 + 2], acc[rt][r0 + 3]));
                if (sg != cur) {
                    flush();
                    cur = sg;
                    run = mg;
                } else {
                    run = fmaxf(run, mg);
                }
            }
        }
    }
    flush();
}

}  // namespace

hipError_t launch_phase1_f32(const Phase1Args& a, const TokenPlan& tp, hipStream_t s)
{
    if (a.nvoc <= 0 || tp.nseg <= 0) return hipSuccess;
    if (tiles_f32_supported(a)) return launch_phase1_tiles_f32(a, tp, s);   // 16-byte aligned rows, m <= 300
    if (tp.group != kGroup) return hipErrorInvalidValue;                  // these kernels take groups of 8 rows
    P1Dev d;
    d.E = (const float*)a.E;
    d.ld = a.ld;
    d.m = a.m;
    d.nkc = (a.m + KC - 1) / KC;
    d.normE = a.normE;
    d.voc_rows = a.voc_rows;
    d.nvoc = a.nvoc;
    d.z_by_position = a.z_by_position;
    d.nvt = (int32_t)((a.nvoc + kTileVocab - 1) / kTileVocab);
    d.nchunks = tp.nchunks;
    d.pofs = tp.pofs;
    d.tok_ids = tp.tok_ids;
    d.tok_hn = tp.tok_hn;
    d.grp_seg = tp.grp_seg;
    d.chunk_seg = tp.chunk_seg;
    d.Z = a.Z;
    d.ldz = a.ldz;
    const int64_t items = (int64_t)d.nvt * d.nchunks;
    const int64_t per_xcd = (items + 7) / 8;
    const int64_t grid = per_xcd * 8;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool vec = (a.m % 4 == 0) && (a.ld % 4 == 0) && (((uintptr_t)a.E & 15) == 0);
    if (d.nkc <= MAXKC) {
        if (vec) k_phase1_f32_regb<true><<<(unsigned)grid, 256, 0, s>>>(d);
        else k_phase1_f32_regb<false><<<(unsigned)grid, 256, 0, s>>>(d);
    } else {
        if (vec) k_phase1_f32_lds<true><<<(unsigned)grid, 256, 0, s>>>(d);
        else k_phase1_f32_lds<false><<<(unsigned)grid, 256, 0, s>>>(d);
    }
    return hipGetLastError();
}

}  // namespace lcrwmd
