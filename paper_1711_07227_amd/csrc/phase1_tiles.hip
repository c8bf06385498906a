// First phase of LC-RWMD (Sec. IV, Fig. 6, many-to-many form): the tile kernel shared by the fp32 and the
// bf16-in / fp32-accumulate paths, for embedding dimensions up to 300.
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
//   * vocabulary operand: NCT x 32 words per wavefront, the whole K extent (304 columns) in registers, loaded
//     once per workgroup;
//   * token operand: tiles of 64 rows x the whole K extent, copied global -> LDS with global_load_lds_dwordx4
//     (no registers), double buffered, ONE barrier per tile; the copy instructions of the next tile are
//     spread over the K steps of the current one so that they never queue up behind each other.
//
// Rows are handled as 16-byte pieces, 8 pieces (one 128-byte cache line) to an "octet": bf16 rows are 5 octets
// (the whole 640-byte packed row), fp32 rows 10 octets (1200 bytes = 75 pieces; the pieces past the end of the row
// re-read piece 74 and meet zeros on the vocabulary side).  One copy instruction moves one octet of 8 rows = 1 KiB:
// the 8 lanes of a row fetch one full line, and lane (row r, slot s) fetches piece s ^ ((r >> 1) & 7), so that the
// later 16-byte LDS reads of 16 consecutive rows of one piece hit all 64 banks.  A tile is 40 KiB (bf16) or 80 KiB
// (fp32); with two buffers, two bf16 workgroups or one fp32 workgroup fill the CU's 160 KiB of LDS exactly.
//
// K step s covers pieces 2 s and 2 s + 1: lane half h multiplies piece 2 s + h of its token row with the same
// piece of its vocabulary word.  bf16: one v_mfma_f32_32x32x16_bf16 per step and tile; fp32: four
// v_mfma_f32_32x32x2_f32 (one per float of the piece).  The LDS reads of step s + 1 are issued before the MFMAs
// of step s and waited for with a partial lgkmcnt.
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
// its own wait insertion drains the whole LDS queue before every use.
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
    int32_t nreal;             // 16-byte pieces that exist in a row; later pieces re-read piece nreal - 1
    int32_t nzero_from;        // fp32: vocabulary values at K index >= this are zero (= m)
    const float* normE;
    const int32_t* voc_rows;
    int64_t nvoc;
    int32_t nvt;
    int32_t nchunks;
    int32_t ntok;              // table mode: number of token rows (tok_ids is readable up to the next multiple of 64 + 64)
    int32_t chunk_tokens;      // table mode: token rows per chunk (a multiple of 64)
    const int32_t* pofs;
    const int32_t* tok_ids;
    const float* tok_hn;
    const int32_t* grp_seg;
    const int32_t* chunk_seg;
    float* Z;
    int64_t ldz;
};

constexpr int ROWS = 64;      // token rows per tile
constexpr int NRT = 2;        // 32-row MFMA tiles per token tile

template <bool BF16>
struct Layout {
    static constexpr int NS = BF16 ? 19 : 38;                 // K steps (pairs of pieces): 304 columns
    static constexpr int NOCT = BF16 ? 5 : 10;                // octets copied per row
    static constexpr int OCT_BYTES = (ROWS / 8) * 1024;       // one octet of all rows of the tile
    static constexpr int TILE_BYTES = NOCT * OCT_BYTES;
    static constexpr int NJOBS = NOCT * (ROWS / 8) / 4;       // copy instructions per wavefront and tile
};

// TABLE = true turns the kernel into the plain pairwise-distance operation C = T o E of Sec. III: no minimum, every
// element sqrt(max(|E_u|^2 + |T_t|^2 - 2 T_t . E_u, 0)) is stored, row t (token) x column u (vocabulary position) with
// pitch ldz.  Tokens are then simply the rows tok_ids[0 .. ntok) cut into chunks of chunk_tokens.
template <bool BF16, int NCT, int WGS_PER_CU, bool TABLE>
__global__ __launch_bounds__(256, WGS_PER_CU) void k_phase1_tiles(P1T p)
{
    using L = Layout<BF16>;
    constexpr int NS = L::NS;
    constexpr int NG = ROWS / 8;               // token groups per tile

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
    int s0 = 0, t0, t1;
    if (TABLE) {
        t0 = chunk * p.chunk_tokens;
        t1 = t0 + p.chunk_tokens < p.ntok ? t0 + p.chunk_tokens : p.ntok;
    } else {
        s0 = p.chunk_seg[chunk];
        const int s1 = p.chunk_seg[chunk + 1];
        if (s0 >= s1) return;
        t0 = p.pofs[s0];
        t1 = p.pofs[s1];
    }
    if (t0 >= t1) return;
    (void)s0;

    const unsigned char* Eb = p.Eb;

    // ---- vocabulary operand -> registers ----
    // Lanes past the end of the vocabulary repeat its last word: they compute and store the same value to the same
    // place as the lane that owns it.  Z is written by position in the vocabulary list (registers are scarce: the
    // row pointer is formed at flush time from the lane id).
    float nEw[NCT];
    f32x4 breg[NS][NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int64_t col = (int64_t)vt * (128 * NCT) + wave * (32 * NCT) + ct * 32 + l31;
        const int64_t colc = col < p.nvoc ? col : p.nvoc - 1;
        const int32_t wid = p.voc_rows ? p.voc_rows[colc] : (int32_t)colc;
        nEw[ct] = p.normE[wid];
        const unsigned char* row = Eb + (int64_t)wid * p.pitch_b;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int piece = 2 * s + half;
            f32x4 x = *reinterpret_cast<const f32x4*>(row + (piece < p.nreal ? piece : p.nreal - 1) * 16);
            if (!BF16) {   // zero beyond the embedding dimension (a re-read piece, or the tail of the last one)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (piece * 4 + t >= p.nzero_from) x[t] = 0.f;
            }
            breg[s][ct] = x;
        }
    }
    if (BF16) {
        // packed rows carry -|row|^2/2 as three bf16 terms in the last K step, upper half, elements 4..6; on the
        // vocabulary side those positions multiply by one
        if (half == 1) {
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                breg[NS - 1][ct][2] = __uint_as_float(0x3F803F80u);   // elements 4, 5 = 1.0
                breg[NS - 1][ct][3] = __uint_as_float(0x00003F80u);   // element 6 = 1.0, element 7 = 0
            }
        }
    }

    // ---- copy jobs of this wavefront ----
    // job J -> octet J / 2, row block (of 8 rows) wave + 4 (J % 2); lane -> row lane / 8, slot lane % 8
    const int lane8 = lane >> 3;                                   // row within an 8-row block; also this lane's token group
    const int pieceO = (lane & 7) ^ ((wave & 1) * 4 + (lane >> 4));
    const uint32_t offO = pieceO * 16;
    // fp32: the last octet reaches past the end of the row (pieces 75..79): re-read the last real piece
    const int last_piece = (L::NOCT - 1) * 8 + pieceO;
    const uint32_t off_last = BF16 ? offO + (L::NOCT - 1) * 128 : (uint32_t)((last_piece < p.nreal ? last_piece : p.nreal - 1) * 16);

    // Word ids of the two token rows this lane copies.  They are fetched when the previous tile's copy jobs have
    // all been issued (one pair of registers serves both) and are multiplied out to byte offsets job by job.
    int32_t wA = 0, wB = 0;
    auto load_words = [&](int tb) {
        const int32_t* t = p.tok_ids + (tb + wave * 8);             // scalar part of the address
        wA = t[lane8];
        wB = t[lane8 + 32];
    };
    const uint32_t pitch32 = (uint32_t)p.pitch_b;     // the host guarantees rows * pitch < 2^32
    // copy job J (compile time) of this wavefront into buffer `lbase`
    auto copy_job = [&](auto j_c, unsigned char* lbase) {
        constexpr int J = decltype(j_c)::value;
        constexpr int oct = J >> 1;
        const uint32_t off = (uint32_t)((J & 1) ? wB : wA) * pitch32 + (oct == L::NOCT - 1 ? off_last : offO + oct * 128);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Eb + off),
                                         (__attribute__((address_space(3))) void*)(lbase + (oct * 8 + (J & 1) * 4 + wave) * 1024),
                                         16, 0, 0);
    };

    // ---- LDS read address of this lane (bytes) ----
    // row block (l31 >> 3), row (l31 & 7), slot (2 k + half) ^ ((l31 >> 1) & 7) for k = s & 3: k enters as an XOR of bits 5..6
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    uint32_t a_oct = lds0 + (l31 >> 3) * 1024 + (l31 & 7) * 128 + ((half ^ ((l31 >> 1) & 7)) * 16);

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
                // both lane halves hold 4 of the 8 rows of every group: exchange and combine
                const unsigned r = __float_as_uint(run[ct]);
                const auto sw = __builtin_amdgcn_permlane32_swap(r, r, false, false);
                const float best = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
                if (half == 0) {
                    int64_t pos = (int64_t)vt * (128 * NCT) + wave * (32 * NCT) + ct * 32 + l31;
                    if (pos >= p.nvoc) pos = p.nvoc - 1;
                    p.Z[pos * p.ldz + cur] = __builtin_amdgcn_sqrtf(fmaxf(nEw[ct] - 2.f * best, 0.f));
                }
            }
        }
    };

    // per-tile side data, fetched one tile ahead: group -> histogram (lane g < NG) and, fp32, -|T|^2/2 per row
    auto load_gs = [&](int tb) { return TABLE ? 0 : (p.grp_seg + (tb >> 3))[lane8]; };   // lanes 8 g .. 8 g + 7 hold group g
    float hn[NRT], hn_next[NRT];
    auto load_hn = [&](int tb, float* h) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) h[rt] = p.tok_hn[tb + rt * 32 + l31];
    };

    // first tile: copy it in one go
    load_words(t0);
    static_for<0, L::NJOBS>([&](auto j_c) { copy_job(j_c, smem); });
    if (t0 + ROWS < t1) load_words(t0 + ROWS);
    int gsv = load_gs(t0);
    if (!BF16) load_hn(t0, hn);
    int buf = 0;

#ifdef DBG_TIMING
    long long tacc[6] = {0, 0, 0, 0, 0, 0};
    long long tprev = clock64();
    const long long dbg_c0 = tprev, dbg_w0 = wall_clock64();
#define DBG_T(k) { long long tn = clock64(); tacc[k] += tn - tprev; tprev = tn; }
#else
#define DBG_T(k)
#endif
    for (int tb = t0; tb < t1; tb += ROWS) {
        __builtin_amdgcn_s_waitcnt(0x0f70);     // vmcnt(0): this wavefront's copies of the tile have landed
        DBG_T(0)
        __syncthreads();                        // ... and everyone's; everyone has left the other buffer
        DBG_T(1)
        const bool more = tb + ROWS < t1;
        unsigned char* next_buf = smem + (buf ^ 1) * L::TILE_BYTES;
        if (more) {
            if (!BF16) load_hn(tb + ROWS, hn_next);
        }
        DBG_T(2)

        // Software pipeline over the K steps: the LDS reads of step s + 1 are issued before the MFMAs of step s,
        // into the other of two fragment register sets; one copy instruction of the next tile rides along every
        // COPY_EVERY steps.
        f32x4 afrag[2][NRT];
        auto issue_reads = [&](auto s_c) {
            constexpr int s = decltype(s_c)::value;
            static_for<0, NRT>([&](auto rt_c) {
                constexpr int rt = decltype(rt_c)::value;
                constexpr int total = (s >> 2) * L::OCT_BYTES + rt * 4096;
                constexpr int win = total / 32768;             // keep the immediate offset below 2^15
                const uint32_t base = (a_oct ^ ((s & 3) << 5)) + win * 32768;
                afrag[s & 1][rt] = lds_read16_nowait<total - win * 32768>(base);
            });
        };
        constexpr int COPY_EVERY = NS / L::NJOBS;
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
#ifndef DBG_NO_COPY
            if constexpr (s % COPY_EVERY == 0 && s / COPY_EVERY < L::NJOBS) {
                if (more) copy_job(std::integral_constant<int, s / COPY_EVERY>{}, next_buf);
            }
            if constexpr (s == COPY_EVERY * (L::NJOBS - 1) + 1) {     // all copy jobs issued: fetch the ids for the tile after next
                if (tb + 2 * ROWS < t1) load_words(tb + 2 * ROWS);
            }
#endif
            __builtin_amdgcn_sched_barrier(0);
        });
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

        if constexpr (TABLE) {
            // every element is a result: register r of row tile rt is token row 32 rt + 8 (r / 4) + 4 half + r % 4
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const int64_t pos = (int64_t)vt * (128 * NCT) + wave * (32 * NCT) + ct * 32 + l31;
                if (pos < p.nvoc) {
                    float* out = p.Z + pos;
#pragma unroll
                    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int row = tb + rt * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                            if (row < t1) out[(int64_t)row * p.ldz] = __builtin_amdgcn_sqrtf(fmaxf(nEw[ct] - 2.f * acc[rt][ct][r], 0.f));
                        }
                }
            }
        }
        // Epilogue: registers 4g'..4g'+3 of row tile rt hold token rows 32 rt + 8 g' + 4 half + {0..3}: group 4 rt + g'.
        int ng = TABLE ? 0 : (t1 - tb) >> 3;
        if (ng > NG) ng = NG;
        // the groups' histograms move to scalar registers; the register then takes the next tile's (one tile ahead)
        int sgs[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) sgs[g] = __builtin_amdgcn_readlane(gsv, 8 * g);
        if (more) gsv = load_gs(tb + ROWS);
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
                const int sg = sgs[g];
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
        if (!BF16) {
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt) hn[rt] = hn_next[rt];
        }
        {   // the other buffer is read next
            a_oct += buf ? -L::TILE_BYTES : L::TILE_BYTES;
        }
        buf ^= 1;
        DBG_T(4)
    }
    if (!TABLE) flush();
#ifdef DBG_TIMING
    if (blockIdx.x == 0 && tid == 0) {
        for (int k = 0; k < 5; ++k) p.Z[k] = (float)tacc[k];
        p.Z[5] = (float)((t1 - t0) / ROWS);
        p.Z[6] = (float)(clock64() - dbg_c0);
        p.Z[7] = (float)(wall_clock64() - dbg_w0);
    }
#endif
}

template <bool BF16, int NCT, int WGS_PER_CU, bool TABLE>
hipError_t launch_tiles(P1T d, hipStream_t s)
{
    d.nvt = (int32_t)((d.nvoc + 128 * NCT - 1) / (128 * NCT));
    const int64_t items = (int64_t)d.nvt * d.nchunks;
    const int64_t grid = (items + 7) / 8 * 8;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const size_t smem = 2 * (size_t)Layout<BF16>::TILE_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_phase1_tiles<BF16, NCT, WGS_PER_CU, TABLE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    k_phase1_tiles<BF16, NCT, WGS_PER_CU, TABLE><<<(unsigned)grid, 256, smem, s>>>(d);
    return hipGetLastError();
}

P1T common_args(const Phase1Args& a, const TokenPlan& tp)
{
    P1T d;
    d.Eb = (const unsigned char*)a.E;
    d.normE = a.normE;
    d.voc_rows = a.voc_rows;
    d.nvoc = a.nvoc;
    d.nvt = 0;
    d.nchunks = tp.nchunks;
    d.ntok = 0;
    d.chunk_tokens = tp.chunk_tokens;
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

// fp32 rows are read in place: 300 values (75 whole 16-byte pieces; the 76th piece of the layout re-reads the 75th)
// in 16-byte aligned rows.  Other shapes take the register-staged kernels of phase1_f32.hip.
bool tiles_f32_supported(const Phase1Args& a)
{
    return a.m == 300 && a.ld % 4 == 0 && (((uintptr_t)a.E) & 15) == 0;
}

hipError_t launch_phase1_tiles_f32(const Phase1Args& a, const TokenPlan& tp, hipStream_t s)
{
    P1T d = common_args(a, tp);
    d.pitch_b = a.ld * 4;
    d.nreal = a.m / 4;
    d.nzero_from = a.m;
    return launch_tiles<false, 2, 1, false>(d, s);
}

// a.E is the packed bf16 copy: 320 values per row, the norm terms in columns 300..302
hipError_t launch_phase1_tiles_bf16(const Phase1Args& a, const TokenPlan& tp, hipStream_t s)
{
    P1T d = common_args(a, tp);
    d.pitch_b = a.ld * 2;
    d.nreal = Layout<true>::NOCT * 8;
    d.nzero_from = 0;
    return launch_tiles<true, 2, 2, false>(d, s);
}

// Pairwise distance table W[t][u] = || E[rows_t[t]] - E[voc_rows[u]] ||, t < ntok, u < a.nvoc, into a.Z with pitch a.ldz.
// tok_ids / tok_hn: the token rows' word ids and -|.|^2/2 (fp32 path), readable up to roundup(ntok, 64) + 64 entries.
bool distance_table_supported(const Phase1Args& a, bool bf16) { return bf16 || tiles_f32_supported(a); }

hipError_t launch_distance_table(const Phase1Args& a, bool bf16, const int32_t* tok_ids, const float* tok_hn,
                                 int64_t ntok, hipStream_t s)
{
    if (a.nvoc <= 0 || ntok <= 0) return hipSuccess;
    if (!distance_table_supported(a, bf16) || ntok > 0x7fffffffLL - 128) return hipErrorNotSupported;
    P1T d;
    d.Eb = (const unsigned char*)a.E;
    d.normE = a.normE;
    d.voc_rows = a.voc_rows;
    d.nvoc = a.nvoc;
    d.nvt = 0;
    d.ntok = (int32_t)ntok;
    // a few thousand work items (vocabulary tiles x chunks of token rows), each chunk 4 .. 64 tiles of 64 rows
    const int64_t nvt = (a.nvoc + 255) / 256;
    const int64_t want_chunks = (4096 + nvt - 1) / nvt;
    int64_t ct = ((ntok + want_chunks - 1) / want_chunks + ROWS - 1) / ROWS * ROWS;
    if (ct < 4 * ROWS) ct = 4 * ROWS;
    if (ct > 64 * ROWS) ct = 64 * ROWS;
    d.chunk_tokens = (int32_t)ct;
    d.nchunks = (int32_t)((ntok + ct - 1) / ct);
    d.pofs = nullptr;
    d.tok_ids = tok_ids;
    d.tok_hn = tok_hn;
    d.grp_seg = nullptr;
    d.chunk_seg = nullptr;
    d.Z = a.Z;
    d.ldz = a.ldz;
    if (bf16) {
        d.pitch_b = a.ld * 2;
        d.nreal = Layout<true>::NOCT * 8;
        d.nzero_from = 0;
        return launch_tiles<true, 2, 2, true>(d, s);
    }
    d.pitch_b = a.ld * 4;
    d.nreal = a.m / 4;
    d.nzero_from = a.m;
    return launch_tiles<false, 2, 1, true>(d, s);
}

}  // namespace lcrwmd
