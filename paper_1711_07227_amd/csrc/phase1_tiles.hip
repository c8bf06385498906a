// First phase of LC-RWMD (Sec. IV, Fig. 6, many-to-many form): the tile kernel shared by the fp32 and the
// bf16-in / fp32-accumulate paths.
//
//   Z[w][j] = sqrt(max(|E_w|^2 - 2 * max_{a in histogram j} (T_a . E_w - |T_a|^2 / 2), 0))
//
// Token rows are the M dimension of the 32x32 MFMA and vocabulary words the N dimension, so a lane owns one
// vocabulary word per column tile and 16 token rows: the minimum over a histogram's tokens is lane-local but
// for one exchange between the lane halves when the histogram ends.  Histograms are padded to groups of 8
// tokens, so each group of 4 accumulator registers belongs to one histogram and the epilogue branches are
// wave-uniform.  The pairwise matrix C = E o T of the paper exists only in accumulators.
//
// Data movement
//   * vocabulary operand: NCT x 32 words per wavefront, the whole K extent in registers (16 bytes per K step
//     and column tile), loaded once per workgroup;
//   * token operand: tiles of NRT x 32 rows x the whole K extent, copied global -> LDS with
//     global_load_lds_dwordx4 (no registers), double buffered, ONE barrier per tile.
// Rows are handled as 16-byte pieces.  A copy instruction moves one "quad" (4 consecutive pieces = 64 bytes)
// of 16 rows: the four lanes of a lane quad fetch 64 contiguous bytes, and lane (row r, slot s) fetches piece
// s ^ ((r >> 2) & 3), so that the 16-byte LDS reads of 16 consecutive rows of one piece hit all 64 banks.
// When the number of pieces is 2 mod 4 the last two pieces form a half quad (32 rows x 32 bytes per
// instruction, swizzled with bit 3 of the row).
//
// K step sigma covers pieces 2 sigma and 2 sigma + 1: lane half h multiplies piece 2 sigma + h of its token row
// with the same piece of its vocabulary word.  bf16: one v_mfma_f32_32x32x16_bf16 per step; fp32: four
// v_mfma_f32_32x32x2_f32 (one per float of the piece).
#include <type_traits>

#include "lcrwmd_internal.h"

namespace lcrwmd {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Compile-time loop: f(std::integral_constant<int, I>{}) for I = B .. E-1.
template <int B, int E, class F>
__device__ inline void static_for(F&& f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// Issue one 16-byte LDS read WITHOUT waiting for it.  The destination registers are written asynchronously; the
// caller waits with s_waitcnt lgkmcnt before using them.  The compiler is deliberately not told about the latency:
// its own wait insertion drains the whole LDS queue before every use, which exposes a full LDS round trip per K step.
template <int OFF>
__device__ inline f32x4 lds_read16_nowait(uint32_t addr)
{
    f32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}

// s_waitcnt that only constrains the LDS/scalar queue: at most N operations still outstanding
#define LCRWMD_WAIT_LGKM(N) __builtin_amdgcn_s_waitcnt(0xC07F | ((N) << 8))

struct P1T {
    const unsigned char* Eb;   // operand rows (fp32: caller's E; bf16: packed copy)
    int64_t pitch_b;           // bytes per row
    int32_t npieces;           // 16-byte pieces copied per row (even)
    int32_t nreal;             // pieces that exist in memory; copies of later pieces re-read piece nreal - 1
    int32_t nzero_from;        // fp32: vocabulary values at K index >= this are zero (= m)
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

// NS > 0 fixes the number of K steps at compile time (the m = 300 case): every guard on the step count folds away
// and a tile's contraction becomes one straight-line block, which lets the LDS reads of the next steps be issued
// under the MFMAs of the current one.  NS = 0 reads the step count from the arguments.
template <bool BF16, int NRT, int NCT, int WGS_PER_CU, int NS>
__global__ __launch_bounds__(256, WGS_PER_CU) void k_phase1_tiles(P1T p)
{
    constexpr int ROWS = NRT * 32;
    constexpr int RB = ROWS / 16;              // 16-row blocks per tile
    constexpr int NR = RB / 4;                 // token rows a lane copies per quad pass (RB = 4 or 8)
    constexpr int QUAD_BYTES = RB * 1024;
    constexpr int MAXS = BF16 ? 19 : 38;       // K steps held in registers (304 columns)
    constexpr int NG = ROWS / 8;               // token groups per tile
    static_assert(RB == 4 || RB == 8, "tiles of 64 or 128 rows");

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: keep it scalar
    const int l31 = lane & 31, half = lane >> 5;

    // Work item -> (chunk, vocabulary tile); each XCD (workgroup id mod 8) gets a contiguous range of items so
    // that its CUs work on the same chunk and share its token rows in that XCD's L2.
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

    const int npieces = NS ? 2 * NS : p.npieces;
    const int nsteps = npieces >> 1;
    const int full_quads = npieces >> 2;
    const bool half_quad = (npieces & 3) != 0;
    const int tbytes = full_quads * QUAD_BYTES + (half_quad ? NRT * 1024 : 0);
    const unsigned char* Eb = p.Eb;

    // ---- vocabulary operand -> registers ----
    bool col_ok[NCT];
    float nEw[NCT];
    float* zout[NCT];
    f32x4 breg[MAXS][NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int64_t col = (int64_t)vt * (128 * NCT) + wave * (32 * NCT) + ct * 32 + l31;
        col_ok[ct] = col < p.nvoc;
        const int64_t colc = col_ok[ct] ? col : p.nvoc - 1;
        const int32_t wid = p.voc_rows ? p.voc_rows[colc] : (int32_t)colc;
        nEw[ct] = p.normE[wid];
        zout[ct] = p.Z + (p.z_by_position ? colc : (int64_t)wid) * p.ldz;
        const unsigned char* row = Eb + (int64_t)wid * p.pitch_b;
#pragma unroll
        for (int s = 0; s < MAXS; ++s) {
            f32x4 x = {0.f, 0.f, 0.f, 0.f};
            if (s < nsteps) {
                const int piece = 2 * s + half;
                x = *reinterpret_cast<const f32x4*>(row + (piece < p.nreal ? piece : p.nreal - 1) * 16);
                if (!BF16) {   // zero beyond the embedding dimension (a re-read piece, or the tail of the last one)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        if (piece * 4 + t >= p.nzero_from) x[t] = 0.f;
                }
            }
            breg[s][ct] = x;
        }
    }
    if (BF16) {
        // packed rows carry -|row|^2/2 as three bf16 terms in the last K step, upper half, elements 4..6; on the
        // vocabulary side those positions multiply by one
        if (half == 1) {
#pragma unroll
            for (int s = 0; s < MAXS; ++s) {
                if (s == nsteps - 1) {
#pragma unroll
                    for (int ct = 0; ct < NCT; ++ct) {
                        breg[s][ct][2] = __uint_as_float(0x3F803F80u);   // elements 4, 5 = 1.0
                        breg[s][ct][3] = __uint_as_float(0x00003F80u);   // element 6 = 1.0, element 7 = 0
                    }
                }
            }
        }
    }

    // ---- copy jobs of this wavefront: job j = 4 i + wave; full quads: quad j / RB, row block j % RB ----
    const int njobs_full = full_quads * RB;
    const int pieceF = (lane & 3) ^ ((lane >> 4) & 3);
    const int pieceH = (lane & 1) ^ ((lane >> 4) & 1);
    const int rowF = wave * 16 + (lane >> 2);           // + 64 for the second row of a lane when RB == 8
    const int rowH = (wave % NRT) * 32 + (lane >> 1);   // half quad: waves 0 .. NRT-1 each copy one 32-row block

    // word ids of the token rows this lane copies, fetched one tile ahead of the copy that uses them
    int32_t wF[NR], wH = 0;
    auto load_words = [&](int tb) {
#pragma unroll
        for (int k = 0; k < NR; ++k) wF[k] = p.tok_ids[tb + rowF + 64 * k];
        if (half_quad) wH = p.tok_ids[tb + rowH];
    };
    // Job i of this wavefront is (quad, row block) = ((4 i + wave) / RB, (4 i + wave) % RB): with RB = 4 that is
    // (i, wave), with RB = 8 it is (i / 2, wave + 4 (i % 2)) - static per i, so the loop unrolls into straight code.
    constexpr int MAXJ = (RB == 4) ? 19 : 18;   // at most 19 full quads (RB = 4) or 9 (RB = 8)
    const int offF = pieceF * 16;
    // pieces past the end of the row (fp32 with an odd piece count) re-read the last real piece
    const int last_piece = (full_quads - 1) * 4 + pieceF;
    const int off_last = (last_piece < p.nreal ? last_piece : p.nreal - 1) * 16;
    auto issue_tile_copy = [&](int buf) {
        const unsigned char* g[NR];
#pragma unroll
        for (int k = 0; k < NR; ++k) g[k] = Eb + (int64_t)wF[k] * p.pitch_b;
        unsigned char* lbase = smem + buf * tbytes + wave * 1024;
#pragma unroll
        for (int i = 0; i < MAXJ; ++i) {
            const int quad = (RB == 4) ? i : (i >> 1);
            if (quad < full_quads) {
                const int rbk = (RB == 4) ? 0 : (i & 1);
                const int off = (quad == full_quads - 1) ? off_last : quad * 64 + offF;
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(g[rbk] + off),
                    (__attribute__((address_space(3))) void*)(lbase + (quad * RB + rbk * 4) * 1024), 16, 0, 0);
            }
        }
        if (half_quad && wave < NRT) {
            int piece = full_quads * 4 + pieceH;
            if (piece >= p.nreal) piece = p.nreal - 1;
            const unsigned char* src = Eb + (int64_t)wH * p.pitch_b + piece * 16;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(lbase + njobs_full * 1024), 16, 0, 0);
        }
    };

    // ---- LDS read offsets of this lane (bytes) for even / odd K steps and for the half quad ----
    const int rsw = (lane >> 2) & 3;
    const int row_off = (((lane >> 4) & 1) * 64 + 4 * (lane & 15)) * 16;
    const int off_even = row_off + ((0 + half) ^ rsw) * 16;
    const int off_odd = row_off + ((2 + half) ^ rsw) * 16;
    const int off_half = (2 * l31 + (half ^ ((lane >> 3) & 1))) * 16;

    f32x16 acc[NRT][NCT];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int cur = -1;
    float run[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) run[ct] = 0.f;
    auto flush = [&]() {
        if (cur >= 0) {
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                // both lane halves hold 8 of the 16 rows of a group pair: exchange and combine
                const unsigned r = __float_as_uint(run[ct]);
                const auto sw = __builtin_amdgcn_permlane32_swap(r, r, false, false);
                const float best = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
                if (half == 0 && col_ok[ct]) zout[ct][cur] = __builtin_amdgcn_sqrtf(fmaxf(nEw[ct] - 2.f * best, 0.f));
            }
        }
    };

    // per-tile side data, fetched one tile ahead: group -> histogram (lane g < NG) and, fp32, -|T|^2/2 per row
    auto load_gs = [&](int tb) { return p.grp_seg[(tb >> 3) + (lane & (NG - 1))]; };
    float hn[NRT], hn_next[NRT];
    auto load_hn = [&](int tb, float* h) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) h[rt] = p.tok_hn[tb + rt * 32 + l31];
    };

    load_words(t0);
    issue_tile_copy(0);
    if (t0 + ROWS < t1) load_words(t0 + ROWS);
    int gsv = load_gs(t0), gsv_next = 0;
    if (!BF16) load_hn(t0, hn);
    int buf = 0;
#ifdef DBG_TIMING
    long long tacc[6] = {0, 0, 0, 0, 0, 0};
    long long tprev = clock64();
#define DBG_T(k) { long long tn = clock64(); tacc[k] += tn - tprev; tprev = tn; }
#else
#define DBG_T(k)
#endif
    for (int tb = t0; tb < t1; tb += ROWS) {
        __builtin_amdgcn_s_waitcnt(0x0f70);     // vmcnt(0): this wavefront's copies of the tile have landed
        DBG_T(0)
        __syncthreads();                        // ... and everyone's; everyone has left the other buffer
        DBG_T(1)
        if (tb + ROWS < t1) {
#ifndef DBG_NO_COPY
            issue_tile_copy(buf ^ 1);                           // word ids were fetched during the previous tile
#endif
            if (tb + 2 * ROWS < t1) load_words(tb + 2 * ROWS);
            gsv_next = load_gs(tb + ROWS);
            if (!BF16) load_hn(tb + ROWS, hn_next);
        }
        DBG_T(2)

        // Software pipeline over the K steps: the LDS reads of step s + 1 are issued before the MFMAs of step s,
        // into the other of two fragment register sets.
        if constexpr (NS > 0) {
            constexpr bool HALFQ = (NS & 1) != 0;                 // 2 NS pieces: a half quad iff NS is odd
            constexpr int FULLQ = (2 * NS) >> 2;
            const uint32_t abase =
                (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem + (uint32_t)(buf * tbytes);
            const uint32_t addr_even = abase + off_even, addr_odd = abase + off_odd, addr_half = abase + off_half;
            f32x4 afrag[2][NRT];
            auto issue_reads = [&](auto s_c) {
                constexpr int s = decltype(s_c)::value;
                constexpr bool in_half = HALFQ && (s == NS - 1);
                constexpr int region = in_half ? FULLQ * QUAD_BYTES : (s >> 1) * QUAD_BYTES;
                constexpr int stride = in_half ? 1024 : 2048;
                static_for<0, NRT>([&](auto rt_c) {
                    constexpr int rt = decltype(rt_c)::value;
                    constexpr int total = region + rt * stride;
                    constexpr int win = total / 32768;             // keep the immediate offset below 2^15
                    const uint32_t base = (in_half ? addr_half : ((s & 1) ? addr_odd : addr_even)) + win * 32768;
                    afrag[s & 1][rt] = lds_read16_nowait<total - win * 32768>(base);
                });
            };
            issue_reads(std::integral_constant<int, 0>{});
            static_for<0, NS>([&](auto s_c) {
                constexpr int s = decltype(s_c)::value;
                if constexpr (s + 1 < NS) {
                    issue_reads(std::integral_constant<int, s + 1>{});
                    LCRWMD_WAIT_LGKM(NRT);          // everything but the reads just issued has arrived
                } else {
                    LCRWMD_WAIT_LGKM(0);
                }
                __builtin_amdgcn_sched_barrier(0);
                const f32x4* a = afrag[s & 1];
                if constexpr (BF16) {
#pragma unroll
                    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                        for (int ct = 0; ct < NCT; ++ct)
                            acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(bf16x8, a[rt]), __builtin_bit_cast(bf16x8, breg[s][ct]),
                                s == 0 ? zero16 : acc[rt][ct], 0, 0, 0);
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                            for (int ct = 0; ct < NCT; ++ct)
                                acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                                    a[rt][t], breg[s][ct][t], (s == 0 && t == 0) ? zero16 : acc[rt][ct], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        } else {
            const unsigned char* A = smem + buf * tbytes;
#pragma unroll
            for (int s = 0; s < MAXS; ++s) {
                if (s < nsteps) {
                    const bool in_half = half_quad && (s == nsteps - 1);
                    const unsigned char* base = in_half ? A + full_quads * QUAD_BYTES + off_half
                                                        : A + (s >> 1) * QUAD_BYTES + ((s & 1) ? off_odd : off_even);
                    const int rstride = in_half ? 1024 : 2048;
                    f32x4 a[NRT];
#pragma unroll
                    for (int rt = 0; rt < NRT; ++rt) a[rt] = *reinterpret_cast<const f32x4*>(base + rt * rstride);
                    if (BF16) {
#pragma unroll
                        for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                            for (int ct = 0; ct < NCT; ++ct)
                                acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                    __builtin_bit_cast(bf16x8, a[rt]), __builtin_bit_cast(bf16x8, breg[s][ct]),
                                    s == 0 ? zero16 : acc[rt][ct], 0, 0, 0);
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t)
#pragma unroll
                            for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                                for (int ct = 0; ct < NCT; ++ct)
                                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                                        a[rt][t], breg[s][ct][t], (s == 0 && t == 0) ? zero16 : acc[rt][ct], 0, 0, 0);
                    }
                }
            }
        }
        if (!BF16) {
            // one more rank-1 step adds -|T_a|^2/2 to every element of token row a
            const float one = half == 0 ? 1.f : 0.f;
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct)
                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(half == 0 ? hn[rt] : 0.f, one, acc[rt][ct], 0, 0, 0);
        }

        DBG_T(3)
        // Epilogue: registers 4g'..4g'+3 of row tile rt hold token rows 32 rt + 8 g' + 4 half + {0..3}: group 4 rt + g'.
        int ng = (t1 - tb) >> 3;
        if (ng > NG) ng = NG;
#ifdef DBG_NO_EPI
        cur = s0;
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) run[ct] = fmaxf(run[ct], acc[rt][ct][r]);
        ng = 0;
#endif
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            if (g < ng) {
                const int sg = __builtin_amdgcn_readlane(gsv, g);
                const int rt = g >> 2, r0 = (g & 3) * 4;
                float mg[NCT];
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct)
                    mg[ct] = fmaxf(fmaxf(acc[rt][ct][r0], acc[rt][ct][r0 + 1]), fmaxf(acc[rt][ct][r0 + 2], acc[rt][ct][r0 + 3]));
                if (sg != cur) {
                    flush();
                    cur = sg;
#pragma unroll
                    for (int ct = 0; ct < NCT; ++ct) run[ct] = mg[ct];
                } else {
#pragma unroll
                    for (int ct = 0; ct < NCT; ++ct) run[ct] = fmaxf(run[ct], mg[ct]);
                }
            }
        }
        gsv = gsv_next;
        if (!BF16) {
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt) hn[rt] = hn_next[rt];
        }
        buf ^= 1;
        DBG_T(4)
    }
    flush();
#ifdef DBG_TIMING
    if (blockIdx.x == 0 && tid == 0) {
        for (int k = 0; k < 5; ++k) p.Z[k] = (float)tacc[k];
        p.Z[5] = (float)((t1 - t0) / ROWS);
    }
#endif
}

template <bool BF16, int NRT, int NCT, int WGS_PER_CU, int NS>
hipError_t launch_tiles(P1T d, hipStream_t s)
{
    d.nvt = (int32_t)((d.nvoc + 128 * NCT - 1) / (128 * NCT));
    const int64_t items = (int64_t)d.nvt * d.nchunks;
    const int64_t grid = (items + 7) / 8 * 8;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const int full_quads = d.npieces >> 2;
    const size_t smem = 2 * ((size_t)full_quads * (NRT * 2 * 1024) + ((d.npieces & 3) ? NRT * 1024 : 0));
    static size_t attr_set = 0;
    if (smem > attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_phase1_tiles<BF16, NRT, NCT, WGS_PER_CU, NS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = smem;
    }
    k_phase1_tiles<BF16, NRT, NCT, WGS_PER_CU, NS><<<(unsigned)grid, 256, smem, s>>>(d);
    return hipGetLastError();
}

P1T common_args(const Phase1Args& a, const TokenPlan& tp)
{
    P1T d;
    d.Eb = (const unsigned char*)a.E;
    d.normE = a.normE;
    d.voc_rows = a.voc_rows;
    d.nvoc = a.nvoc;
    d.z_by_position = a.z_by_position;
    d.nvt = 0;
    d.nchunks = tp.nchunks;
    d.pofs = tp.pofs;
    d.tok_ids = tp.tok_ids;
    d.tok_hn = tp.tok_hn;
    d.grp_seg = tp.grp_seg;
    d.chunk_seg = tp.chunk_seg;
    d.Z = a.Z;
    d.ldz = a.ldz;
    return d;
}

}  // namespace

bool tiles_f32_supported(const Phase1Args& a)
{
    return a.m <= 300 && a.m % 4 == 0 && a.ld % 4 == 0 && (((uintptr_t)a.E) & 15) == 0;
}

hipError_t launch_phase1_tiles_f32(const Phase1Args& a, const TokenPlan& tp, hipStream_t s)
{
    P1T d = common_args(a, tp);
    d.pitch_b = a.ld * 4;
    d.nreal = a.m / 4;
    d.npieces = (d.nreal + 1) & ~1;
    d.nzero_from = a.m;
#ifdef DBG_F32_NCT1
    if (d.npieces == 76) return launch_tiles<false, 2, 1, 1, 38>(d, s);
#endif
    if (d.npieces == 76) return launch_tiles<false, 2, 2, 1, 38>(d, s);   // m = 300
    return launch_tiles<false, 2, 2, 1, 0>(d, s);
}

// a.E is the packed bf16 copy, a.ld its pitch in elements; nsteps K steps of 16 are in use
hipError_t launch_phase1_tiles_bf16(const Phase1Args& a, int32_t nsteps, const TokenPlan& tp, hipStream_t s)
{
    P1T d = common_args(a, tp);
    d.pitch_b = a.ld * 2;
    d.npieces = 2 * nsteps;
    d.nreal = d.npieces;
    d.nzero_from = 0;
    if (nsteps == 19) return launch_tiles<true, 2, 2, 2, 19>(d, s);       // m = 300
    return launch_tiles<true, 2, 2, 2, 0>(d, s);
}

}  // namespace lcrwmd
