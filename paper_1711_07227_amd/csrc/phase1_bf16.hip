// First phase of LC-RWMD with bf16 operands and fp32 accumulation (Sec. IV, Fig. 6, many-to-many form).
//
// Same mathematics and work decomposition as the fp32 kernel:
//   Z[w][j] = sqrt(max(|E_w|^2 - 2 * max_{a in histogram j} (T_a . E_w - |T_a|^2 / 2), 0))
// with token rows as the M dimension of v_mfma_f32_32x32x16_bf16, so that a lane owns one vocabulary word
// and the minimum over a histogram's tokens stays lane-local.
//
// Packed operand (pack kernel below): one row per word, `pitch` bf16 values (a multiple of 32, i.e. whole
// 64-byte lines): columns [0, m) hold the embedding rounded to bf16 (round-to-nearest-even), then zeros,
// and the three columns just before the end of the last 16-wide K step hold -|row|^2/2 split into three
// bf16 terms.  A word used as a TOKEN brings these along; for a word used as VOCABULARY the kernel
// overwrites the same three positions of its register copy with 1.0, so the contraction itself adds the
// -|T_a|^2/2 term and the epilogue is a plain maximum.
//
// Data movement: the vocabulary operand of a wavefront (64 words x K) lives in registers for the whole
// workgroup; token tiles (128 rows x full K, 76 KiB) are copied global -> LDS by global_load_lds_dwordx4
// without passing through registers, double buffered, one barrier per tile.  Each copy instruction moves
// 16 rows x one 64-byte line: the four lanes of a quad fetch one line (coalesced), in an order that is
// XOR-swizzled with the row so that the later 16-byte LDS reads of 16 consecutive rows hit 64 distinct banks.
#include "lcrwmd_internal.h"

namespace lcrwmd {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kMaxSteps = 19;            // K steps of 16 held in registers: m + 4 <= 304
constexpr int kVocabPerWave = 64;
constexpr int kVocabPerBlock = 256;      // 4 wavefronts
constexpr int kRows = kTileTokens;       // 128 token rows per tile

__device__ inline uint16_t f32_to_bf16_rne(float x)
{
    uint32_t b = __float_as_uint(x);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}
__device__ inline float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// One wavefront per row.
__global__ __launch_bounds__(256) void k_pack_bf16(const void* __restrict__ E, int is_bf16, int64_t v, int32_t m,
                                                   int64_t ld, int32_t pitch, int32_t norm_col,
                                                   uint16_t* __restrict__ packed, float* __restrict__ normE)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= v) return;
    uint16_t* out = packed + w * pitch;
    float s = 0.f;
    for (int t = lane; t < pitch; t += 64) {
        uint16_t h = 0;
        if (t < m) {
            h = is_bf16 ? reinterpret_cast<const uint16_t*>(E)[w * ld + t]
                        : f32_to_bf16_rne(reinterpret_cast<const float*>(E)[w * ld + t]);
            const float x = bf16_to_f32(h);
            s = fmaf(x, x, s);
        }
        if (t < norm_col || t >= norm_col + 3) out[t] = h;
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) {
        normE[w] = s;
        const float hn = -0.5f * s;
        const uint16_t h0 = f32_to_bf16_rne(hn);
        const float r1 = hn - bf16_to_f32(h0);
        const uint16_t h1 = f32_to_bf16_rne(r1);
        const uint16_t h2 = f32_to_bf16_rne(r1 - bf16_to_f32(h1));
        out[norm_col] = h0;
        out[norm_col + 1] = h1;
        out[norm_col + 2] = h2;
    }
}

struct P1B {
    const uint16_t* Ep;       // packed rows
    int32_t pitch;            // bf16 elements per packed row (multiple of 32)
    int32_t nsteps;           // K steps of 16
    const float* normE;
    const int32_t* voc_rows;
    int64_t nvoc;
    int32_t z_by_position;
    int32_t nvt;
    int32_t nchunks;
    const int32_t* pofs;
    const int32_t* tok_ids;
    const int32_t* grp_seg;
    const int32_t* chunk_seg;
    float* Z;
    int64_t ldz;
};

// LDS tile: full 64-byte lines first (8 KiB per line index: 8 blocks of 16 rows x 64 B), then, when the
// number of 16-byte pieces per row is not a multiple of 4, one half line (4 blocks of 32 rows x 32 B).
__host__ __device__ inline int tile_bytes(int nsteps)
{
    const int pieces = 2 * nsteps;
    return (pieces / 4) * 8192 + ((pieces & 3) ? 4096 : 0);
}

__global__ __launch_bounds__(256, 1) void k_phase1_bf16(P1B p)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

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

    const int nsteps = p.nsteps;
    const int full_lines = (2 * nsteps) >> 2;          // 64-byte lines with all four pieces in use
    const bool half_line = ((2 * nsteps) & 3) != 0;    // then pieces 4*full_lines, +1 form a half line
    const int tbytes = tile_bytes(nsteps);
    const int64_t pitch_b = (int64_t)p.pitch * 2;
    const unsigned char* Eb = reinterpret_cast<const unsigned char*>(p.Ep);

    // ---- this lane's two vocabulary words and their operand registers ----
    int64_t colc[2];
    bool col_ok[2];
    float nEw[2];
    float* zout[2];
    bf16x8 breg[kMaxSteps][2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
        const int64_t col = (int64_t)vt * kVocabPerBlock + wave * kVocabPerWave + ct * 32 + l31;
        col_ok[ct] = col < p.nvoc;
        colc[ct] = col_ok[ct] ? col : p.nvoc - 1;
        const int32_t wid = p.voc_rows ? p.voc_rows[colc[ct]] : (int32_t)colc[ct];
        nEw[ct] = p.normE[wid];
        zout[ct] = p.Z + (p.z_by_position ? colc[ct] : (int64_t)wid) * p.ldz;
        const unsigned char* row = Eb + (int64_t)wid * pitch_b + half * 16;
#pragma unroll
        for (int s = 0; s < kMaxSteps; ++s) {
            if (s < nsteps) breg[s][ct] = *reinterpret_cast<const bf16x8*>(row + s * 32);
            else breg[s][ct] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
    }
    // the vocabulary side of the three norm columns is 1.0: last K step, upper half, elements 4..6
    if (half == 1) {
#pragma unroll
        for (int s = 0; s < kMaxSteps; ++s) {
            if (s == nsteps - 1) {
#pragma unroll
                for (int ct = 0; ct < 2; ++ct) {
                    breg[s][ct][4] = (__bf16)1.0f;
                    breg[s][ct][5] = (__bf16)1.0f;
                    breg[s][ct][6] = (__bf16)1.0f;
                    breg[s][ct][7] = (__bf16)0.0f;
                }
            }
        }
    }

    // ---- copy instructions of this wavefront: instruction j = 4 i + wave ----
    // full lines: j = line * 8 + row_block (16 rows); lane -> row (lane >> 2), piece (lane & 3) ^ ((lane >> 4) & 3)
    // half line : j = full_lines * 8 + row_block32; lane -> row (lane >> 1), piece (lane & 1) ^ ((lane >> 4) & 1)
    const int njobs_full = full_lines * 8;
    const int njobs = njobs_full + (half_line ? 4 : 0);
    const int rowA = (wave & 3) * 16 + (lane >> 2);            // row block alternates between wave and wave + 4
    const int rowB = rowA + 64;
    const int pieceF = (lane & 3) ^ ((lane >> 4) & 3);
    const int rowH = wave * 32 + (lane >> 1);                  // half line: row block = j - njobs_full = wave
    const int pieceH = (lane & 1) ^ ((lane >> 4) & 1);

    auto issue_tile_copy = [&](int tb, int buf) {
        const int32_t wA = p.tok_ids[tb + rowA], wB = p.tok_ids[tb + rowB], wH = p.tok_ids[tb + rowH];
        const unsigned char* gA = Eb + (int64_t)wA * pitch_b + pieceF * 16;
        const unsigned char* gB = Eb + (int64_t)wB * pitch_b + pieceF * 16;
        const unsigned char* gH = Eb + (int64_t)wH * pitch_b + full_lines * 64 + pieceH * 16;
        unsigned char* lbase = smem + buf * tbytes;
        // job j = 4 i + wave: row block (j & 7) = wave (i even) or wave + 4 (i odd); line = j >> 3 = i >> 1
        for (int i = 0; 4 * i + wave < njobs_full; ++i) {
            const int j = 4 * i + wave;
            const unsigned char* g = ((i & 1) ? gB : gA) + (j >> 3) * 64;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                             (__attribute__((address_space(3))) void*)(lbase + j * 1024), 16, 0, 0);
        }
        if (half_line)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gH,
                                             (__attribute__((address_space(3))) void*)(lbase + (njobs_full + wave) * 1024),
                                             16, 0, 0);
        (void)njobs;
    };

    // ---- LDS read offsets of this lane (bytes), for even and odd K steps and for the half line ----
    const int rsw = (lane >> 2) & 3;
    const int off_even = ((((lane >> 4) & 1) * 64) + 4 * (lane & 15) + ((0 + half) ^ rsw)) * 16;
    const int off_odd = ((((lane >> 4) & 1) * 64) + 4 * (lane & 15) + ((2 + half) ^ rsw)) * 16;
    const int off_half = (2 * l31 + (half ^ ((lane >> 3) & 1))) * 16;

    f32x16 acc[4][2];
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int cur = -1;
    float run[2] = {0.f, 0.f};
    auto flush = [&]() {
        if (cur >= 0) {
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) {
                const float other = __shfl_xor(run[ct], 32);
                const float best = fmaxf(run[ct], other);
                if (half == 0 && col_ok[ct]) zout[ct][cur] = sqrtf(fmaxf(nEw[ct] - 2.f * best, 0.f));
            }
        }
    };

    issue_tile_copy(t0, 0);
    int buf = 0;
    for (int tb = t0; tb < t1; tb += kRows) {
        const int gsv = p.grp_seg[(tb >> 3) + (lane & 15)];
        __builtin_amdgcn_s_waitcnt(0x0f70);     // vmcnt(0): this wavefront's copies have landed in LDS
        __syncthreads();                        // everyone's have, and everyone left the other buffer
        if (tb + kRows < t1) issue_tile_copy(tb + kRows, buf ^ 1);

        const unsigned char* A = smem + buf * tbytes;
#pragma unroll
        for (int s = 0; s < kMaxSteps; ++s) {
            if (s < nsteps) {
                const bool in_half_line = half_line && (s == nsteps - 1);
                const unsigned char* base =
                    in_half_line ? A + full_lines * 8192 + off_half : A + (s >> 1) * 8192 + ((s & 1) ? off_odd : off_even);
                const int rstride = in_half_line ? 1024 : 2048;
                bf16x8 a[4];
#pragma unroll
                for (int rt = 0; rt < 4; ++rt) a[rt] = *reinterpret_cast<const bf16x8*>(base + rt * rstride);
#pragma unroll
                for (int rt = 0; rt < 4; ++rt)
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct)
                        acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rt], breg[s][ct],
                                                                              s == 0 ? zero16 : acc[rt][ct], 0, 0, 0);
            }
        }

        int ng = (t1 - tb) >> 3;
        if (ng > 16) ng = 16;
#pragma unroll
        for (int g = 0; g < 16; ++g) {
            if (g < ng) {
                const int sg = __builtin_amdgcn_readlane(gsv, g);
                const int rt = g >> 2, r0 = (g & 3) * 4;
                float mg[2];
#pragma unroll
                for (int ct = 0; ct < 2; ++ct)
                    mg[ct] = fmaxf(fmaxf(acc[rt][ct][r0], acc[rt][ct][r0 + 1]), fmaxf(acc[rt][ct][r0 + 2], acc[rt][ct][r0 + 3]));
                if (sg != cur) {
                    flush();
                    cur = sg;
                    run[0] = mg[0];
                    run[1] = mg[1];
                } else {
                    run[0] = fmaxf(run[0], mg[0]);
                    run[1] = fmaxf(run[1], mg[1]);
                }
            }
        }
        buf ^= 1;
    }
    flush();
}

}  // namespace

// K steps needed for m values plus the three norm columns, and the packed row pitch in elements.
static int32_t steps_for(int32_t m) { return (m + 4 + 15) / 16; }   // the last four columns of the last step are reserved
bool bf16_supported(int32_t m) { return steps_for(m) <= kMaxSteps; }
int32_t bf16_pitch(int32_t m) { return ((steps_for(m) * 16 + 31) / 32) * 32; }
size_t pack_bf16_bytes(int64_t v, int32_t m) { return (size_t)v * (size_t)bf16_pitch(m) * 2; }

hipError_t launch_pack_bf16(const void* E, lcrwmd_dtype dtype, int64_t v, int32_t m, int64_t ld, void* packed,
                            float* normE, hipStream_t s)
{
    if (v <= 0) return hipSuccess;
    if (steps_for(m) > kMaxSteps) return hipErrorNotSupported;
    const int32_t norm_col = steps_for(m) * 16 - 4;
    k_pack_bf16<<<(unsigned)((v + 3) / 4), 256, 0, s>>>(E, dtype == LCRWMD_BF16 ? 1 : 0, v, m, ld, bf16_pitch(m), norm_col,
                                                       (uint16_t*)packed, normE);
    return hipGetLastError();
}

hipError_t launch_phase1_bf16(const Phase1Args& a, const TokenPlan& tp, hipStream_t s)
{
    if (a.nvoc <= 0 || tp.nseg <= 0) return hipSuccess;
    if (steps_for(a.m) > kMaxSteps) return hipErrorNotSupported;
    P1B d;
    d.Ep = (const uint16_t*)a.E;
    d.pitch = bf16_pitch(a.m);
    d.nsteps = steps_for(a.m);
    d.normE = a.normE;
    d.voc_rows = a.voc_rows;
    d.nvoc = a.nvoc;
    d.z_by_position = a.z_by_position;
    d.nvt = (int32_t)((a.nvoc + kVocabPerBlock - 1) / kVocabPerBlock);
    d.nchunks = tp.nchunks;
    d.pofs = tp.pofs;
    d.tok_ids = tp.tok_ids;
    d.grp_seg = tp.grp_seg;
    d.chunk_seg = tp.chunk_seg;
    d.Z = a.Z;
    d.ldz = a.ldz;
    const int64_t items = (int64_t)d.nvt * d.nchunks;
    const int64_t grid = (items + 7) / 8 * 8;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const size_t smem = 2 * (size_t)tile_bytes(d.nsteps);
    static size_t attr_set = 0;
    if (smem > attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_phase1_bf16),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = smem;
    }
    k_phase1_bf16<<<(unsigned)grid, 256, smem, s>>>(d);
    return hipGetLastError();
}

}  // namespace lcrwmd
