// First phase of LC-RWMD (Sec. IV, Fig. 6, many-to-many form): the tile kernels shared by the fp32, the split-bf16 and
// the bf16-in / fp32-accumulate paths, for embedding dimensions up to 300.
//
//   Z[w][j] = sqrt(max(|E_w|^2 - 2 * max_{a in histogram j} (T_a . E_w - |T_a|^2 / 2), 0))
//
// Two kernels: k_phase1_pingpong computes Z (contraction + minimum per histogram, nothing else leaves the
// accumulators); k_distance_table is the plain pairwise-distance operation C = T o E of Sec. III, every element stored,
// for the table form of the bound.  They share the layout described here.
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
//   * token operand: tiles of ROWS rows x the whole K extent, copied global -> LDS with global_load_lds_dwordx4
//     (no registers) into a ring of NBUF buffers, ONE barrier per tile; the copy instructions of the tile
//     NBUF - 1 ahead are spread over the K steps of the current one so that they never queue up behind each
//     other.  fp32: 64-row tiles, 2 buffers (a tile is ~44k MFMA clocks, far more than the memory latency);
//     bf16 table kernel: 32-row tiles, 4 buffers (a tile is only ~1.2k MFMA clocks: copies have to be three tiles ahead).
//
// Rows are handled as 16-byte pieces, 8 pieces (one 128-byte cache line) to an "octet": bf16 rows are 5 octets
// (the whole 640-byte packed row), fp32 rows 10 octets (1200 bytes = 75 pieces; the pieces past the end of the row
// re-read piece 74 and meet zeros on the vocabulary side).  One copy instruction moves one octet of 8 rows = 1 KiB:
// the 8 lanes of a row fetch one full line, and lane (row r, slot s) fetches piece s ^ ((r >> 1) & 7), so that the
// later 16-byte LDS reads of 16 consecutive rows of one piece hit all 64 banks.  A tile is 20 KiB (bf16) or 80 KiB
// (fp32); two bf16 workgroups (4 buffers each) or one fp32 workgroup (2 buffers) fill the CU's 160 KiB of LDS exactly.
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
    int32_t ntok;              // k_distance_table: number of token rows (tok_ids is readable up to the next multiple of 64 + 64)
    int32_t chunk_tokens;      // k_distance_table: token rows per chunk (a multiple of 64)
    const int32_t* pofs;
    const int32_t* tok_ids;
    const float* tok_hn;
    const int32_t* grp_seg;
    const int32_t* chunk_seg;
    float* Z;
    int64_t ldz;
    // Optional map of the entries that may need a second look (k_phase1_pingpong only): word close_pitch * j + slice
    // holds, for histogram j and the 32 * NCT vocabulary positions of one wavefront (slice = that wavefront's number in
    // vocabulary order), one bit per lane: set where the squared distance came out below a quarter of the word's squared
    // norm - a pair of close or equal words, for which the norm expansion is not accurate.  Every word is written.
    uint64_t* close_bits;
    int64_t close_pitch;
    int32_t park;              // bf16 k_phase1_pingpong: collect four histograms' results per lane in LDS and store 16 bytes
};

// Arithmetic of the contraction.
//   F32:  fp32 operands, v_mfma_f32_32x32x2_f32.
//   BF16: operands rounded to bf16, v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//   X3:   every fp32 operand value x is split into two bf16 terms, hi = bf16(x) and lo = bf16(x - hi), and the product
//         of two values is taken as hi*hi + hi*lo + lo*hi (three bf16 MFMAs, fp32 accumulation; the lo*lo term, 2^-16
//         relative, is dropped).  The operand rows hold the 304 hi values followed by the 304 lo values: the row has
//         the shape of an fp32 row (76 pieces), K step s < 19 is the hi piece pair and step s + 19 its lo pair.
enum : int { kF32 = 0, kBF16 = 1, kX3 = 2 };

// Tile shape per path: ROWS token rows (NRT 32-row MFMA tiles) and NBUF LDS buffers.
template <int MODE>
struct Layout {
    static constexpr int ROWS = MODE == kBF16 ? 32 : 64;
    static constexpr int NRT = ROWS / 32;
    static constexpr int NBUF = MODE == kBF16 ? 4 : 2;
    static constexpr int PD = NBUF - 1;                       // tiles between a copy and its use
    static constexpr int LA = MODE == kBF16 ? 3 : 1;           // K-loop iterations between an LDS read and its use
    static constexpr int NS = MODE == kBF16 ? 19 : 38;         // pairs of 16-byte pieces per operand row (registers, LDS reads)
    static constexpr int NITER = MODE == kX3 ? 19 : NS;        // K-loop iterations (X3: a hi and a lo pair per iteration)
    static constexpr int NOCT = MODE == kBF16 ? 5 : 10;        // octets copied per row
    static constexpr int OCT_BYTES = (ROWS / 8) * 1024;       // one octet of all rows of the tile
    static constexpr int TILE_BYTES = NOCT * OCT_BYTES;
    static constexpr int NJOBS = NOCT * (ROWS / 8) / 4;       // copy instructions per wavefront and tile
};
constexpr int kMaxRows = 64;

// The plain pairwise-distance operation C = T o E of Sec. III: every element sqrt(max(|E_u|^2 + |T_t|^2 - 2 T_t . E_u, 0))
// is stored, row t (token) x column u (vocabulary position) with pitch ldz.  Tokens are the rows tok_ids[0 .. ntok) cut
// into chunks of chunk_tokens.  One workgroup of four wavefronts per (vocabulary tile of 128 NCT words, chunk).
template <int MODE, int NCT, int WGS_PER_CU, bool WIDE>
__global__ __launch_bounds__(256, WGS_PER_CU) void k_distance_table(P1T p)
{
    using L = Layout<MODE>;
    constexpr bool BF16 = MODE == kBF16, X3 = MODE == kX3;
    constexpr int NS = L::NS, NITER = L::NITER;
    constexpr int ROWS = L::ROWS, NRT = L::NRT, NBUF = L::NBUF, PD = L::PD;

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: keep it scalar
    const int l31 = lane & 31, half = lane >> 5;

    // Work item -> (chunk, vocabulary tile).  XCD x (workgroup id mod 8) takes, of chunk c, the vocabulary tiles
    // congruent to x - c mod 8, chunk after chunk: whatever the number of tiles and the chunks' lengths, all XCDs
    // carry the same load (the residues rotate), and the CUs of an XCD work on the same chunk at the same time,
    // sharing its token rows in that XCD's L2.  Eight consecutive chunks hold exactly nvt items of every XCD.
    int chunk, vt;
    {
        const int xcd = blockIdx.x & 7;
        const int64_t slot = blockIdx.x >> 3;
        const int64_t period = slot / p.nvt;
        int rem = (int)(slot - period * p.nvt);
        chunk = -1;
        vt = 0;
#pragma unroll 1
        for (int k = 0; k < 8; ++k) {
            const int r = (xcd - k) & 7;                          // residue of this XCD in chunk 8 * period + k
            const int n = r < p.nvt ? (p.nvt - r + 7) >> 3 : 0;
            if (rem < n) { chunk = (int)(period * 8) + k; vt = r + 8 * rem; break; }
            rem -= n;
        }
        if (chunk < 0 || chunk >= p.nchunks) return;
    }
    const int t0 = chunk * p.chunk_tokens;
    const int t1 = t0 + p.chunk_tokens < p.ntok ? t0 + p.chunk_tokens : p.ntok;
    if (t0 >= t1) return;

    const unsigned char* Eb = p.Eb;

    // ---- vocabulary operand -> registers ----
    // Lanes past the end of the vocabulary repeat its last word and store nothing.
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
            if (!BF16 && !X3) {   // zero beyond the embedding dimension (a re-read piece, or the tail of the last one)
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
    // job J -> octet J / NRT, row block (of 8 rows) wave + 4 (J % NRT); lane -> row lane / 8, slot lane % 8
    const int lane8 = lane >> 3;                                   // row within an 8-row block
    // Source offsets in units of U bytes: 16-byte pieces when the operand rows span 4 GiB or more (32 bits then reach
    // 64 GiB; the host checks it), bytes otherwise.
    constexpr uint32_t U = WIDE ? 16 : 1, PIECE = 16 / U;
    const int pieceO = (lane & 7) ^ ((wave & 1) * 4 + (lane >> 4));
    const uint32_t offO = pieceO * PIECE;
    // fp32: the last octet reaches past the end of the row (pieces 75..79): re-read the last real piece
    const int last_piece = (L::NOCT - 1) * 8 + pieceO;
    const uint32_t off_last = (BF16 || X3) ? offO + (L::NOCT - 1) * 8 * PIECE : (uint32_t)(last_piece < p.nreal ? last_piece : p.nreal - 1) * PIECE;

    // Word ids of the two token rows this lane copies.  They are fetched when the previous tile's copy jobs have
    // all been issued (one pair of registers serves both) and are multiplied out to byte offsets job by job.
    int32_t wA = 0, wB = 0;
    auto load_words = [&](int tb) {
        const int32_t* t = p.tok_ids + (tb + wave * 8);             // scalar part of the address
        wA = t[lane8];
        if (NRT == 2) wB = t[lane8 + 32];
    };
    const uint32_t pitchU = (uint32_t)(p.pitch_b / U);     // the host guarantees rows * pitchU < 2^32
    // copy job J (compile time) of this wavefront into buffer `lbase`
    auto copy_job = [&](auto j_c, unsigned char* lbase) {
        constexpr int J = decltype(j_c)::value;
        constexpr int oct = J / NRT, blk = J % NRT;
        const uint32_t off = (uint32_t)(blk ? wB : wA) * pitchU + (oct == L::NOCT - 1 ? off_last : offO + oct * 8 * PIECE);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(WIDE ? Eb + ((uint64_t)off << 4) : Eb + off),
                                         (__attribute__((address_space(3))) void*)(lbase + (oct * (ROWS / 8) + blk * 4 + wave) * 1024),
                                         16, 0, 0);
    };

    // ---- LDS read address of this lane (bytes) ----
    // row block (l31 >> 3), row (l31 & 7), slot (2 k + half) ^ ((l31 >> 1) & 7) for k = s & 3: k enters as an XOR of bits 5..6
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    const uint32_t a_oct0 = lds0 + (l31 >> 3) * 1024 + (l31 & 7) * 128 + ((half ^ ((l31 >> 1) & 7)) * 16);

    f32x16 acc[NRT][NCT];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // per-tile side data, fetched one tile ahead: fp32, -|T|^2/2 per row
    float hn[NRT], hn_next[NRT];
    auto load_hn = [&](int tb, float* h) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) h[rt] = p.tok_hn[tb + rt * 32 + l31];
    };

    // the first PD tiles: copy each in one go
    static_for<0, PD>([&](auto k_c) {
        constexpr int k = decltype(k_c)::value;
        if (t0 + k * ROWS < t1) {
            load_words(t0 + k * ROWS);
            static_for<0, L::NJOBS>([&](auto j_c) { copy_job(j_c, smem + k * L::TILE_BYTES); });
        }
    });
    if (t0 + PD * ROWS < t1) load_words(t0 + PD * ROWS);
    if (!BF16) load_hn(t0, hn);
    int buf = 0;                               // ring position of the tile being multiplied

    for (int tb = t0; tb < t1; tb += ROWS) {
        // This wavefront's copies of the tile have landed.  Vector memory operations complete in issue order and the
        // copies of the PD - 1 later tiles were issued after this tile's: while those are all still to come, at most
        // (PD - 1) * NJOBS operations may remain outstanding; at the end of the chunk everything is waited for.
        if (PD > 1 && tb + (PD - 1) * ROWS < t1) __builtin_amdgcn_s_waitcnt(0x0f70 | ((PD - 1) * L::NJOBS));
        else __builtin_amdgcn_s_waitcnt(0x0f70);
        __syncthreads();                        // ... and everyone's; everyone has left the buffer refilled next
        const bool more = tb + ROWS < t1;
        const bool more_copy = tb + PD * ROWS < t1;
        const int buf_copy = buf == 0 ? NBUF - 1 : buf - 1;          // = (buf + PD) mod NBUF
        unsigned char* next_buf = smem + buf_copy * L::TILE_BYTES;
        const uint32_t a_oct = a_oct0 + buf * L::TILE_BYTES;
        if (more) {
            if (!BF16) load_hn(tb + ROWS, hn_next);
        }

        // Software pipeline over the K steps: the LDS reads of step s + LA are issued before the MFMAs of step s,
        // into a ring of LA + 1 fragment register sets (LA steps of MFMAs have to cover the LDS latency: a bf16 step
        // is only 64 MFMA clocks); one copy instruction of a later tile rides along every COPY_EVERY steps.
        constexpr int LA = L::LA;
        constexpr int NF = X3 ? 2 : 1;                   // fragments per iteration and row tile (X3: hi and lo)
        f32x4 afrag[LA + 1][NRT][NF];
        auto issue_reads = [&](auto s_c) {
            constexpr int s = decltype(s_c)::value;
            static_for<0, NRT>([&](auto rt_c) {
                constexpr int rt = decltype(rt_c)::value;
                static_for<0, NF>([&](auto f_c) {
                    constexpr int step = s + decltype(f_c)::value * 19;            // piece pair read
                    constexpr int total = (step >> 2) * L::OCT_BYTES + rt * 4096;
                    constexpr int win = total / 32768;             // keep the immediate offset below 2^15
                    const uint32_t base = (a_oct ^ ((step & 3) << 5)) + win * 32768;
                    afrag[s % (LA + 1)][rt][decltype(f_c)::value] = lds_read16_nowait<total - win * 32768>(base);
                });
            });
        };
        constexpr int COPY_EVERY = NITER >= L::NJOBS ? NITER / L::NJOBS : 1;
        static_for<0, LA>([&](auto s_c) { issue_reads(s_c); });
        static_for<0, NITER>([&](auto s_c) {
            constexpr int s = decltype(s_c)::value;
            if constexpr (WGS_PER_CU > 1) {
                // Two wavefronts share a SIMD's matrix pipe.  Priority rises through the K loop, so of two wavefronts
                // that multiply at the same time the one further along wins the pipe and pulls ahead: the pair
                // settles into one multiplying while the other runs its epilogue, instead of both doing the same.
                if constexpr (s == 0) __builtin_amdgcn_s_setprio(0);
                if constexpr (s == NITER / 3) __builtin_amdgcn_s_setprio(1);
                if constexpr (s == (2 * NITER) / 3) __builtin_amdgcn_s_setprio(2);
            }
            if constexpr (s + LA < NITER) issue_reads(std::integral_constant<int, s + LA>{});
            {
                constexpr int later = (NITER - 1 - s < LA ? NITER - 1 - s : LA) * NRT * NF;     // reads issued after step s's
                LCRWMD_WAIT_LGKM(later);
            }
            __builtin_amdgcn_sched_barrier(0);
            const auto& a = afrag[s % (LA + 1)];
            if constexpr (X3) {
                // hi*hi, hi*lo, lo*hi: the four accumulators take turns, so dependent MFMAs are four apart
                static_for<0, 3>([&](auto term_c) {
                    constexpr int term = decltype(term_c)::value;
                    constexpr int fa = term == 2 ? 1 : 0, sb = term == 1 ? s + 19 : s;
#pragma unroll
                    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                        for (int ct = 0; ct < NCT; ++ct)
                            acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(bf16x8, a[rt][fa]), __builtin_bit_cast(bf16x8, breg[sb][ct]),
                                (s == 0 && term == 0) ? zero16 : acc[rt][ct], 0, 0, 0);
                });
            } else if constexpr (BF16) {
#pragma unroll
                for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                    for (int ct = 0; ct < NCT; ++ct)
                        acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, a[rt][0]), __builtin_bit_cast(bf16x8, breg[s][ct]),
                            s == 0 ? zero16 : acc[rt][ct], 0, 0, 0);
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                        for (int ct = 0; ct < NCT; ++ct)
                            acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                                a[rt][0][t], breg[s][ct][t], (s == 0 && t == 0) ? zero16 : acc[rt][ct], 0, 0, 0);
            }
            // copy jobs of a later tile, spread over the iterations (X3: 20 jobs over 19 iterations, the last takes two)
            static_for<0, L::NJOBS>([&](auto j_c) {
                constexpr int j = decltype(j_c)::value;
                constexpr int at = j * COPY_EVERY < NITER ? j * COPY_EVERY : NITER - 1;
                if constexpr (at == s) {
                    if (more_copy) copy_job(j_c, next_buf);
                }
            });
            if constexpr (s == ((L::NJOBS - 1) * COPY_EVERY < NITER ? (L::NJOBS - 1) * COPY_EVERY + 1 : NITER) ||
                          (s == NITER - 1 && (L::NJOBS - 1) * COPY_EVERY + 1 >= NITER)) {
                // all copy jobs issued: fetch the ids for the next tile to copy
                if (tb + (PD + 1) * ROWS < t1) load_words(tb + (PD + 1) * ROWS);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        if constexpr (WGS_PER_CU > 1) __builtin_amdgcn_s_setprio(3);      // the stores go first
        if (!BF16) {
            // one more rank-1 step adds -|T_a|^2/2 to every element of token row a
            const float one = half == 0 ? 1.f : 0.f;
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct)
                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(half == 0 ? hn[rt] : 0.f, one, acc[rt][ct], 0, 0, 0);
        }

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
        if (!BF16) {
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt) hn[rt] = hn_next[rt];
        }
        buf = buf == NBUF - 1 ? 0 : buf + 1;
    }
}

// ---------------------------------------------------------------------------------------------------------------
// bf16 first phase, "ping-pong" form.  A bf16 tile is so short (76 MFMAs, ~2.4k clocks) that neither its epilogue nor
// the barrier around it can be hidden behind the MFMAs of the same wavefront.  Here one workgroup of EIGHT wavefronts
// owns a CU: two groups of four (one wavefront of each group per SIMD), each group covering 256 vocabulary words, both
// reading the same token tiles.  The groups run half a period apart: while one group multiplies a tile, the other one
// runs the epilogue of the tile it multiplied before and issues its share of the copies; a workgroup barrier ends
// every half period.  The matrix pipe of a SIMD is then always owned by exactly one wavefront, and everything that is
// not an MFMA happens in the other wavefront's shadow.
//
// Token tiles: 64 rows, the layout of the kernel above, in a ring of four buffers (160 KiB).  The five copy
// instructions a wavefront contributes to tile t + 3 ride along its K loop over tile t.  It waits for its own copies
// of tile t + 2 at the end of that K loop with a partial vmcnt: vector memory operations complete in issue order,
// and the five copy instructions of tile t + 3 were issued later, so "at most five outstanding" means the copies of
// tile t + 2 (and everything older) have landed.  The barrier that follows publishes them.
//
// The same schedule serves the fp32 and the split-bf16 arithmetic (one 32-word column tile per wavefront instead of
// two, so that eight wavefronts fit the register file; 80 KiB tiles in two buffers, copies one tile ahead): their
// tiles are long enough to hide a barrier, but not the copy instructions' issue stalls and the epilogue, which cost
// a wavefront that owns its SIMD alone a tenth of its time.
template <int MODE>
struct PP {
    static constexpr int ROWS = 64, NRT = 2;
    static constexpr int NCT = MODE == kBF16 ? 2 : 1;          // 32-word column tiles per wavefront
    static constexpr int NS = MODE == kBF16 ? 19 : 38;         // pairs of 16-byte pieces per operand row
    static constexpr int NITER = MODE == kF32 ? 38 : 19;       // K-loop iterations
    static constexpr int NF = MODE == kX3 ? 2 : 1;             // fragments per iteration and row tile (hi, lo)
    static constexpr int NOCT = MODE == kBF16 ? 5 : 10;
    static constexpr int NBUF = MODE == kBF16 ? 4 : 2;
    static constexpr int PD = NBUF - 1;
    static constexpr int OCT_BYTES = (ROWS / 8) * 1024, TILE_BYTES = NOCT * OCT_BYTES;
    // Rows per group = the padding of a histogram's token list.  Groups of 4 cost sixteen epilogue steps per tile
    // instead of eight; measured on Medium that pays for the split-bf16 arithmetic (-3 %) and costs the other two
    // (fp32 +1.3 %, and the bf16 epilogue no longer fits in the other group's K loop), so only the split form uses it.
    static constexpr int G = MODE == kX3 ? 4 : 8;
    static constexpr int NG = ROWS / G;
    static constexpr int WG_COLS = 2 * 4 * NCT * 32;           // vocabulary words per workgroup
    static constexpr int COPY_EVERY = NITER / NOCT >= 1 ? NITER / NOCT : 1;
};

// Workgroup barrier WITHOUT the memory fences of __syncthreads(): a fence would wait for every outstanding vector
// memory operation, i.e. for the copies just issued for a tile three periods away and for the stores of Z.  What a
// barrier has to order here is waited for explicitly: LDS reads with lgkmcnt(0) at the end of a K loop, a
// wavefront's own copies with vmcnt(0) at the start of its next epilogue.
__device__ inline void pp_barrier() { __builtin_amdgcn_s_barrier(); }

//
// The per-tile side tables (word ids of the rows to copy, histogram of every group of 8 rows) are read with uniform
// addresses through restrict-qualified arguments, i.e. as scalar loads: they are then not part of the vector memory
// queue whose order the copy waits rely on, and they cost no vector registers.
// WIDE: the operand rows span 4 GiB or more: copy offsets are then counted in 16-byte pieces (32 bits reach 64 GiB)
// instead of bytes, at the price of a shift per copy instruction (measured: 9 % of the bf16 kernel's time, which is
// why the byte form stays the default).
template <int MODE, bool WIDE>
__global__ __launch_bounds__(512, 1) void k_phase1_pingpong(P1T p, const int32_t* __restrict__ tok_ids,
                                                            const int32_t* __restrict__ grp_seg)
{
    using C = PP<MODE>;
    constexpr bool BF16 = MODE == kBF16, X3 = MODE == kX3, F32 = MODE == kF32;
    constexpr int ROWS = C::ROWS, NRT = C::NRT, NCT = C::NCT, NS = C::NS, NITER = C::NITER, NF = C::NF, NOCT = C::NOCT;
    constexpr int NBUF = C::NBUF, PD = C::PD, OCT_BYTES = C::OCT_BYTES, TILE_BYTES = C::TILE_BYTES, NG = C::NG, G = C::G;
    constexpr int WG_COLS = C::WG_COLS;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // 0..7
    const int grp = wave >> 2;                                    // 0: multiplies first; 1: half a period later
    const int l31 = lane & 31, half = lane >> 5;

    // Work: the (vocabulary tile, chunk) pairs in vocabulary-major order, cut into gridDim.x equal runs, one per
    // workgroup (the grid is one workgroup per CU).  Chunks are short and end at histogram boundaries; a run of
    // chunks of one vocabulary tile is one uninterrupted stream of token tiles, so the load is balanced to within a
    // chunk and the vocabulary operand is reloaded only where a run crosses into the next vocabulary tile.
    // Workgroups of one XCD (workgroup id mod 8) take neighbouring runs.
    const int64_t total = (int64_t)p.nvt * p.nchunks;
    const int64_t wg = (int64_t)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    int64_t item = wg * total / gridDim.x;
    const int64_t item_end = (wg + 1) * total / gridDim.x;

    const unsigned char* Eb = p.Eb;
    const int lane8 = lane >> 3;
    const int pieceO = (lane & 7) ^ ((wave & 1) * 4 + (lane >> 4));
    // Source offsets in units of U bytes (the host checks that 32 bits suffice)
    constexpr uint32_t U = WIDE ? 16 : 1, PIECE = 16 / U;
    const uint32_t offO = (uint32_t)pieceO * PIECE;
    // fp32 rows end inside the last octet (pieces 75..79 do not exist): those lanes re-read the last real piece,
    // which meets zeros on the vocabulary side
    const int last_piece = (NOCT - 1) * 8 + pieceO;
    const uint32_t off_last = (uint32_t)(last_piece < p.nreal ? last_piece : p.nreal - 1) * PIECE - offO;
    const uint32_t pitchU = (uint32_t)(p.pitch_b / U);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
    const uint32_t a_oct0 = lds0 + (l31 >> 3) * 1024 + (l31 & 7) * 128 + ((half ^ ((l31 >> 1) & 7)) * 16);
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    while (item < item_end) {
    const int vt = (int)(item / p.nchunks);
    const int c0 = (int)(item - (int64_t)vt * p.nchunks);
    const int c1 = (int)(item_end - item < p.nchunks - c0 ? c0 + (item_end - item) : p.nchunks);
    item += c1 - c0;
    const int t0 = p.pofs[p.chunk_seg[c0]], t1 = p.pofs[p.chunk_seg[c1]];
    if (t0 >= t1) continue;
    const int64_t col0 = (int64_t)vt * WG_COLS + wave * (32 * NCT);      // first vocabulary position of this wavefront

    // ---- vocabulary operand -> registers (lanes past the end repeat the last word) ----
    float nEw[NCT];
    f32x4 breg[NS][NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int64_t col = col0 + ct * 32 + l31;
        const int64_t colc = col < p.nvoc ? col : p.nvoc - 1;
        const int32_t wid = p.voc_rows ? p.voc_rows[colc] : (int32_t)colc;
        nEw[ct] = p.normE[wid];
        const unsigned char* row = Eb + (int64_t)wid * p.pitch_b;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int piece = 2 * s + half;
            f32x4 x = *reinterpret_cast<const f32x4*>(row + (piece < p.nreal ? piece : p.nreal - 1) * 16);
            if (F32) {        // zero beyond the embedding dimension (a re-read piece, or the tail of the last one)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (piece * 4 + t >= p.nzero_from) x[t] = 0.f;
            }
            breg[s][ct] = x;
        }
    }
    if (BF16 && half == 1) {          // the three -|row|^2/2 terms of the token side multiply by one here
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            breg[NS - 1][ct][2] = __uint_as_float(0x3F803F80u);
            breg[NS - 1][ct][3] = __uint_as_float(0x00003F80u);
        }
    }

    // ---- copies: wavefront w moves row block w (rows 8 w .. 8 w + 7) of a tile, one octet per instruction ----
    // word ids of the 8 rows this wavefront copies (uniform), and this lane's pick
    struct Ids { int32_t v[8]; };
    auto load_ids = [&](int tb) {
        Ids r;
        const int32_t* t = tok_ids + (tb + wave * 8);
#pragma unroll
        for (int k = 0; k < 8; ++k) r.v[k] = t[k];
        return r;
    };
    // offset of this lane's piece of its row, from the row block's 8 word ids
    auto row_offset = [&](const Ids& ids) {
        // lane l < 8 takes id l, then every lane fetches the id of its row from lane (row within the block)
        int32_t spread = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) asm("v_writelane_b32 %0, %1, %2" : "+v"(spread) : "s"(ids.v[k]), "n"(k));
        const int32_t wA = __builtin_amdgcn_ds_bpermute(lane8 << 2, spread);
        return (uint32_t)wA * pitchU + offO;
    };
    auto copy_octet = [&](auto o_c, uint32_t off, unsigned char* lbase) {
        constexpr int oct = decltype(o_c)::value;
        const uint32_t o = off + ((F32 && oct == NOCT - 1) ? off_last : (uint32_t)(oct * 8) * PIECE);
        // bf16: pieces 38 and 39 of a row (columns 304..319) are never multiplied; the copies leave their 32 bytes per
        // row alone, and those bytes - 8 KiB over the four tile buffers - are where results are parked (see flush)
        if (!BF16 || oct != NOCT - 1 || pieceO < 6)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(WIDE ? Eb + ((uint64_t)o << 4) : Eb + o),
                                             (__attribute__((address_space(3))) void*)(lbase + (oct * (ROWS / 8) + wave) * 1024),
                                             16, 0, 0);
    };
    auto copy_tile = [&](const Ids& ids, unsigned char* lbase) {
        const uint32_t off = row_offset(ids);
        static_for<0, NOCT>([&](auto o_c) { copy_octet(o_c, off, lbase); });
    };

    f32x16 acc[NRT][NCT];
    // Running maximum of the histogram being walked (`cur`), per column tile and lane half; a histogram's value is
    // complete when the next one starts.  The running maximum is updated with selects; the only branch per group of 8
    // rows is the one around the store (taken when a histogram ends).
    int cur = -1;
    float run[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) run[ct] = 0.f;
    const float nEsel = (NCT == 2 && half) ? nEw[NCT - 1] : nEw[0];
    float* zrow;
    {
        // two column tiles: lower lanes own tile 0, upper lanes tile 1; one: both halves own the same 32 words
        int64_t pos = col0 + (NCT == 2 ? lane : l31);
        if (pos >= p.nvoc) pos = p.nvoc - 1;
        zrow = p.Z + pos * p.ldz;
    }
    // Store the value of histogram `cur`.  One exchange hands the lower lanes both halves' maxima of column tile 0
    // and the upper lanes those of column tile 1, so one store serves 64 words (with a single column tile both
    // halves end up with the same value and store it to the same place).
    uint64_t* const bits = p.close_bits ? p.close_bits + ((int64_t)vt * 8 + wave) : nullptr;      // this wavefront's slice
    // bf16: a lane's results of four consecutive histograms are collected in 16 bytes of LDS of its own and leave as
    // one aligned 16-byte store.  (One 4-byte store per word and histogram reaches the memory system as a write of its
    // own - the L2s are swept by the token tiles before a sector's neighbours arrive - and at this kernel's pace those
    // requests cost it a tenth of its time.)  The 16 bytes: wavefront w, lane l -> tile buffer w mod 4, token row l,
    // piece 38 + w / 4 of that row, which no copy writes and no MFMA reads.  park_q: first histogram of the quad being
    // collected, counted from a 16-byte boundary of Z's rows; park_mask: which of its four slots are filled.
    const bool parking = BF16 && p.park;
    const int zoff = (int)(((uintptr_t)p.Z >> 2) & 3);
    float* const park_slot = reinterpret_cast<float*>(smem + (wave & 3) * TILE_BYTES + (4 * (ROWS / 8) + (lane >> 3)) * 1024 +
                                                      (lane & 7) * 128 + (((6 + (wave >> 2)) ^ ((lane >> 1) & 7)) * 16));
    int park_q = -4;
    unsigned park_mask = 0;
    auto unpark = [&]() {          // stores whatever is collected, slot by slot (only where a run starts or ends inside a quad)
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (park_mask & (1u << t)) zrow[park_q - zoff + t] = park_slot[t];
        park_mask = 0;
    };
    auto flush = [&]() {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(run[0]), __float_as_uint(run[NCT - 1]), false, false);
        const float best = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        const float d2 = nEsel - 2.f * best;
        const float z = __builtin_amdgcn_sqrtf(fmaxf(d2, 0.f));
        if (parking) {
            const int a = cur + zoff, q = a & ~3;
            if (q != park_q) {
                if (park_mask) unpark();
                park_q = q;
            }
            park_slot[a & 3] = z;
            park_mask |= 1u << (a & 3);
            if (park_mask == 15u) {
                *reinterpret_cast<f32x4*>(zrow + (q - zoff)) = *reinterpret_cast<const f32x4*>(park_slot);
                park_mask = 0;
            }
        } else {
            zrow[cur] = z;
        }
        if (bits) {
            const uint64_t close = __ballot(4.f * d2 < nEsel);
            if (lane == 0) bits[(int64_t)cur * p.close_pitch] = close;
        }
    };

    struct Grp { int32_t v[NG]; };
    auto load_gs = [&](int tb) {
        Grp r;
        const int32_t* g = grp_seg + tb / G;
#pragma unroll
        for (int k = 0; k < NG; ++k) r.v[k] = g[k];
        return r;
    };

    // ---- the first PD tiles ----
    static_for<0, PD>([&](auto k_c) {
        constexpr int k = decltype(k_c)::value;
        if (t0 + k * ROWS < t1) copy_tile(load_ids(t0 + k * ROWS), smem + k * TILE_BYTES);
    });
    // copies of tile t + PD ride along the K loop of tile t; their source offsets are formed one epilogue earlier
    uint32_t off_next = row_offset(load_ids(t0 + PD * ROWS < t1 ? t0 + PD * ROWS : t0));
    Ids ids_next = load_ids(t0 + (PD + 1) * ROWS < t1 ? t0 + (PD + 1) * ROWS : t0);
    Grp grp_next = load_gs(t0);
    // fp32 and split bf16: -|T_a|^2/2 of this lane's two token rows, added by a rank-1 fp32 MFMA step per tile
    float hn[NRT] = {}, hn_next[NRT] = {};
    auto load_hn = [&](int tb, float* h) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) h[rt] = p.tok_hn[tb + rt * 32 + l31];
    };
    if (!BF16) load_hn(t0, hn);
    __builtin_amdgcn_s_waitcnt(0x0f70);        // vmcnt(0): this wavefront's share of the first tiles has landed
    pp_barrier();
    if (grp == 1) pp_barrier();                // the second group starts half a period later

    // The epilogue of a tile: histogram maxima of its groups, the stores of the histograms that end in it, the source
    // offsets of the copies two K loops ahead and the scalar table loads for the epilogue after this one.
    // Rows 8 j .. 8 j + 3 of a 32-row tile sit in accumulator registers 4 j .. 4 j + 3 of the lower lane half, rows
    // 8 j + 4 .. 8 j + 7 in the same registers of the upper half.  A group of 8 rows is those registers in both halves;
    // groups of 4 are walked in row order and only the half that owns a group adds it to its running maximum (the
    // store combines the two halves either way).
    auto epilogue = [&](int tb) {
        int ng = (t1 - tb) / G;
        if (ng > NG) ng = NG;
        const Grp sgsv = grp_next;
        const Ids ids = ids_next;
        const int32_t* sgs = sgsv.v;
        if (tb + (PD + 1) * ROWS < t1) off_next = row_offset(ids);
        // the next epilogue's tables: requested only now, so that the wait for the lane exchange above does not
        // include them, and early enough to be back before the next K loop counts its LDS reads
        __builtin_amdgcn_sched_barrier(0);
        if (tb + ROWS < t1) grp_next = load_gs(tb + ROWS);
        if (tb + (PD + 2) * ROWS < t1) ids_next = load_ids(tb + (PD + 2) * ROWS);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const bool live = g < ng;                      // groups past the end of the chunk are someone else's
            const int sg = live ? sgs[g] : cur;
            const bool is_new = sg != cur;
            const int rt = G == 4 ? g >> 3 : g >> 2, r0 = G == 4 ? ((g & 7) >> 1) * 4 : (g & 3) * 4;
            const bool mine = G == 8 || (g & 1) == half;
            if (is_new && cur >= 0) flush();
            cur = sg;
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const float mg = fmaxf(fmaxf(acc[rt][ct][r0], acc[rt][ct][r0 + 1]), fmaxf(acc[rt][ct][r0 + 2], acc[rt][ct][r0 + 3]));
                run[ct] = fmaxf((live && mine) ? mg : -INFINITY, is_new ? -INFINITY : run[ct]);
            }
        }
    };

    // One loop iteration = [epilogue of the previous tile] [first LDS reads of this tile] barrier [K loop] barrier.
    // The reads are issued BEFORE the barrier that starts the K loop, so the matrix pipe does not wait for the LDS
    // latency at the start of every half period; they are legal there because every wavefront waits, at the end of
    // its K loop over tile t, for its copies of tile t + 2 (not t + 1): a tile is complete in LDS, and published by a
    // barrier, a full period before its first read.
    int buf = 0;
    for (int tb = t0; tb < t1; tb += ROWS) {
        if (tb > t0) epilogue(tb - ROWS);
        const uint32_t a_oct = a_oct0 + buf * TILE_BYTES;
        const bool more_copy = tb + PD * ROWS < t1;
        unsigned char* copy_buf = smem + (buf == 0 ? NBUF - 1 : buf - 1) * TILE_BYTES;   // (buf + PD) mod NBUF: the tile before this one is done with
        // Two fragment register sets: the reads of iteration s + 1 are issued before the MFMAs of iteration s.
        f32x4 afrag[2][NRT][NF];
        auto issue_reads = [&](auto s_c) {
            constexpr int s = decltype(s_c)::value;
            static_for<0, NRT>([&](auto rt_c) {
                constexpr int rt = decltype(rt_c)::value;
                static_for<0, NF>([&](auto f_c) {
                    constexpr int step = s + decltype(f_c)::value * 19;            // piece pair read (split bf16: hi, lo)
                    constexpr int total = (step >> 2) * OCT_BYTES + rt * 4096;
                    constexpr int win = total / 32768;                              // keep the immediate offset below 2^15
                    const uint32_t base = (a_oct ^ ((step & 3) << 5)) + win * 32768;
                    afrag[s & 1][rt][decltype(f_c)::value] = lds_read16_nowait<total - win * 32768>(base);
                });
            });
        };
        // With copies three tiles ahead a tile is published a full period before its first read, and the first reads
        // may precede the barrier; with copies one tile ahead (fp32, split bf16) the other group's share of this tile
        // is published by this very barrier.
        if (PD >= 3) issue_reads(std::integral_constant<int, 0>{});
        if (tb > t0) pp_barrier();              // ends the half period of the epilogue above
        if (PD < 3) issue_reads(std::integral_constant<int, 0>{});
        if (!BF16 && tb + ROWS < t1) load_hn(tb + ROWS, hn_next);     // before this K loop's copies: never waits for them
        // ================= multiply =================
        static_for<0, NITER>([&](auto s_c) {
            constexpr int s = decltype(s_c)::value;
            if constexpr (s + 1 < NITER) {
                issue_reads(std::integral_constant<int, s + 1>{});
                LCRWMD_WAIT_LGKM(NRT * NF);
            } else {
                LCRWMD_WAIT_LGKM(0);
            }
            __builtin_amdgcn_sched_barrier(0);
            const auto& a = afrag[s & 1];
            if constexpr (X3) {
                // hi*hi, hi*lo, lo*hi; the accumulators take turns, so dependent MFMAs are two apart
                static_for<0, 3>([&](auto term_c) {
                    constexpr int term = decltype(term_c)::value;
                    constexpr int fa = term == 2 ? 1 : 0, sb = term == 1 ? s + 19 : s;
#pragma unroll
                    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                        for (int ct = 0; ct < NCT; ++ct)
                            acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(bf16x8, a[rt][fa]), __builtin_bit_cast(bf16x8, breg[sb][ct]),
                                (s == 0 && term == 0) ? zero16 : acc[rt][ct], 0, 0, 0);
                });
            } else if constexpr (BF16) {
#pragma unroll
                for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                    for (int ct = 0; ct < NCT; ++ct)
                        acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, a[rt][0]), __builtin_bit_cast(bf16x8, breg[s][ct]),
                            s == 0 ? zero16 : acc[rt][ct], 0, 0, 0);
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                        for (int ct = 0; ct < NCT; ++ct)
                            acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                                a[rt][0][t], breg[s][ct][t], (s == 0 && t == 0) ? zero16 : acc[rt][ct], 0, 0, 0);
            }
            // a copy instruction stalls at issue for a while: in the MFMAs' shadow of the other group it is free
            if constexpr (s % C::COPY_EVERY == 1 % C::COPY_EVERY && s / C::COPY_EVERY < NOCT) {
                if (more_copy) copy_octet(std::integral_constant<int, s / C::COPY_EVERY>{}, off_next, copy_buf);
            }
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
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt) hn[rt] = hn_next[rt];
        }
        // This wavefront's copies have landed: with copies three tiles ahead, those of the tile after next (the five of
        // the tile beyond were issued later, see the head of the kernel); with copies one tile ahead, all of them.
        if (PD >= 3 && tb + PD * ROWS < t1) __builtin_amdgcn_s_waitcnt(0x0f70 | NOCT);
        else __builtin_amdgcn_s_waitcnt(0x0f70);
        pp_barrier();
        buf = buf == NBUF - 1 ? 0 : buf + 1;
    }
    epilogue(t1 - 1 - ((t1 - 1 - t0) % ROWS));      // the last tile's
    pp_barrier();
    if (grp == 0) pp_barrier();             // both groups pass the same number of barriers; nobody reads LDS any more
    if (cur >= 0) flush();
    if (park_mask) unpark();
    }   // runs of this workgroup
}

bool rows_within_4gib(int64_t rows, int64_t pitch_bytes) { return rows * pitch_bytes < ((int64_t)1 << 32); }

template <int MODE, int NCT, int WGS_PER_CU, bool WIDE>
hipError_t launch_tiles_w(P1T d, hipStream_t s);

template <int MODE, int NCT, int WGS_PER_CU>
hipError_t launch_tiles(P1T d, int64_t erows, hipStream_t s)
{
    return rows_within_4gib(erows, d.pitch_b) ? launch_tiles_w<MODE, NCT, WGS_PER_CU, false>(d, s)
                                              : launch_tiles_w<MODE, NCT, WGS_PER_CU, true>(d, s);
}

template <int MODE, int NCT, int WGS_PER_CU, bool WIDE>
hipError_t launch_tiles_w(P1T d, hipStream_t s)
{
    d.nvt = (int32_t)((d.nvoc + 128 * NCT - 1) / (128 * NCT));
    const int64_t grid = 8 * (int64_t)d.nvt * ((d.nchunks + 7) / 8);       // per XCD: nvt items in every 8 chunks
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const size_t smem = (size_t)Layout<MODE>::NBUF * (size_t)Layout<MODE>::TILE_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_distance_table<MODE, NCT, WGS_PER_CU, WIDE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    k_distance_table<MODE, NCT, WGS_PER_CU, WIDE><<<(unsigned)grid, 256, smem, s>>>(d);
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
    d.close_bits = a.close_bits;
    d.close_pitch = 0;
    d.park = a.ldz % 4 == 0 ? 1 : 0;      // 16-byte stores need rows of Z that keep the alignment of the first one
    return d;
}

}  // namespace

// fp32 rows are read in place: 300 values (75 whole 16-byte pieces; the 76th piece of the layout re-reads the 75th)
// in 16-byte aligned rows.  Other shapes take the register-staged kernels of phase1_f32.hip.
int phase1_group_x3() { return PP<kX3>::G; }

// Shape of the map of close pairs the contraction kernel of a mode writes: vocabulary positions per 64-bit word (the
// lower 32 bits count where it is 32) and words per histogram.
int close_bits_slice(int mode) { return mode == 1 ? 64 : 32; }
int64_t close_bits_pitch(int mode, int64_t nvoc)
{
    const int64_t wg = mode == 1 ? PP<kBF16>::WG_COLS : PP<kF32>::WG_COLS;
    return (nvoc + wg - 1) / wg * 8;
}

// The copies address operand rows with 32-bit offsets: bytes while the rows span less than 4 GiB, 16-byte pieces
// (a slower variant of the kernels) up to 64 GiB.
bool tiles_rows_addressable(int64_t rows, int64_t pitch_bytes) { return pitch_bytes % 16 == 0 && rows * (pitch_bytes / 16) < ((int64_t)1 << 32); }

bool tiles_f32_supported(const Phase1Args& a)
{
    return a.m == 300 && a.ld % 4 == 0 && (((uintptr_t)a.E) & 15) == 0 && tiles_rows_addressable(a.erows, a.ld * 4);
}

// One workgroup of eight wavefronts per CU (it takes all of a CU's LDS), fewer when there is less work than that.
template <int MODE, bool WIDE>
hipError_t launch_pingpong_w(P1T d, int num_cu, hipStream_t s);

template <int MODE>
hipError_t launch_pingpong(P1T d, int64_t erows, int num_cu, hipStream_t s)
{
    return rows_within_4gib(erows, d.pitch_b) ? launch_pingpong_w<MODE, false>(d, num_cu, s) : launch_pingpong_w<MODE, true>(d, num_cu, s);
}

template <int MODE, bool WIDE>
hipError_t launch_pingpong_w(P1T d, int num_cu, hipStream_t s)
{
    using C = PP<MODE>;
    d.nvt = (int32_t)((d.nvoc + C::WG_COLS - 1) / C::WG_COLS);
    d.close_pitch = (int64_t)d.nvt * 8;
    const int64_t total = (int64_t)d.nvt * d.nchunks;
    int64_t grid = num_cu > 8 ? num_cu / 8 * 8 : 8;
    while (grid > 8 && grid > total) grid -= 8;
    const size_t smem = (size_t)C::NBUF * C::TILE_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_phase1_pingpong<MODE, WIDE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    k_phase1_pingpong<MODE, WIDE><<<(unsigned)grid, 512, smem, s>>>(d, d.tok_ids, d.grp_seg);
    return hipGetLastError();
}

hipError_t launch_phase1_tiles_f32(const Phase1Args& a, const TokenPlan& tp, hipStream_t s)
{
    P1T d = common_args(a, tp);
    d.pitch_b = a.ld * 4;
    d.nreal = a.m / 4;
    d.nzero_from = a.m;
    if (tp.group != PP<kF32>::G) return hipErrorInvalidValue;      // the token plan was padded for another kernel
    if (!tiles_f32_supported(a)) return hipErrorInvalidValue;
    return launch_pingpong<kF32>(d, a.erows, a.num_cu, s);
}

// a.E is the split copy: 640 bf16 per row (304 hi, 304 lo, zeros); norms and -|T|^2/2 stay fp32 as in the fp32 path
hipError_t launch_phase1_tiles_x3(const Phase1Args& a, const TokenPlan& tp, hipStream_t s)
{
    P1T d = common_args(a, tp);
    d.pitch_b = a.ld * 2;
    d.nreal = Layout<kX3>::NOCT * 8;
    d.nzero_from = 0;
    if (tp.group != PP<kX3>::G) return hipErrorInvalidValue;      // the token plan was padded for another kernel
    if (!tiles_rows_addressable(a.erows, d.pitch_b)) return hipErrorInvalidValue;
    return launch_pingpong<kX3>(d, a.erows, a.num_cu, s);
}

// a.E is the packed bf16 copy: 320 values per row, the norm terms in columns 300..302
hipError_t launch_phase1_tiles_bf16(const Phase1Args& a, const TokenPlan& tp, int num_cu, hipStream_t s)
{
    P1T d = common_args(a, tp);
    d.pitch_b = a.ld * 2;
    d.nreal = Layout<kBF16>::NOCT * 8;
    d.nzero_from = 0;
    if (tp.group != PP<kBF16>::G) return hipErrorInvalidValue;      // the token plan was padded for another kernel
    if (!tiles_rows_addressable(a.erows, d.pitch_b)) return hipErrorInvalidValue;
    return launch_pingpong<kBF16>(d, a.erows, num_cu, s);
}

// Pairwise distance table W[t][u] = || E[rows_t[t]] - E[voc_rows[u]] ||, t < ntok, u < a.nvoc, into a.Z with pitch a.ldz.
// tok_ids / tok_hn: the token rows' word ids and -|.|^2/2 (fp32 path), readable up to roundup(ntok, 64) + 64 entries.
bool distance_table_supported(const Phase1Args& a, int mode)
{
    return mode != 0 ? tiles_rows_addressable(a.erows, a.ld * 2) : tiles_f32_supported(a);
}

hipError_t launch_distance_table(const Phase1Args& a, int mode, const int32_t* tok_ids, const float* tok_hn,
                                 int64_t ntok, hipStream_t s)
{
    if (a.nvoc <= 0 || ntok <= 0) return hipSuccess;
    if (!distance_table_supported(a, mode) || ntok > 0x7fffffffLL - 128) return hipErrorNotSupported;
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
    int64_t ct = ((ntok + want_chunks - 1) / want_chunks + kMaxRows - 1) / kMaxRows * kMaxRows;
    if (ct < 4 * kMaxRows) ct = 4 * kMaxRows;
    if (ct > 64 * kMaxRows) ct = 64 * kMaxRows;
    d.chunk_tokens = (int32_t)ct;
    d.nchunks = (int32_t)((ntok + ct - 1) / ct);
    d.pofs = nullptr;
    d.tok_ids = tok_ids;
    d.tok_hn = tok_hn;
    d.grp_seg = nullptr;
    d.chunk_seg = nullptr;
    d.Z = a.Z;
    d.ldz = a.ldz;
    d.close_bits = nullptr;
    d.close_pitch = 0;
    d.park = 0;
    if (mode == 1) {
        d.pitch_b = a.ld * 2;
        d.nreal = Layout<kBF16>::NOCT * 8;
        d.nzero_from = 0;
        return launch_tiles<kBF16, 2, 2>(d, a.erows, s);
    }
    if (mode == 2) {
        d.pitch_b = a.ld * 2;
        d.nreal = Layout<kX3>::NOCT * 8;
        d.nzero_from = 0;
        return launch_tiles<kX3, 2, 1>(d, a.erows, s);
    }
    d.pitch_b = a.ld * 4;
    d.nreal = a.m / 4;
    d.nzero_from = a.m;
    return launch_tiles<kF32, 2, 1>(d, a.erows, s);
}

}  // namespace lcrwmd
