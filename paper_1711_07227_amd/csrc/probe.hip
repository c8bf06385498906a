// Diagnostic, not part of the method: what the matrix cores of the device sustain for the first phase's MFMA
// shapes, as a function of the operand data and of where the A operand comes from.  The dense-MFMA peak figures
// assume the full shader clock; under sustained bf16 MFMA load on data that toggles the part lowers its clock
// (power limit), so the rate a contraction kernel can reach on real embeddings is below the spec-sheet peak whatever
// its instruction stream looks like.  lcrwmd_probe_mfma measures that ceiling: a loop of nothing but MFMAs on
// operands held in registers (or with the A operand re-read from LDS every two MFMAs, the rate of the first-phase
// kernel), timed with events; the shader clock follows from the ratio of the cycle counter to the wall-clock counter.
// lcrwmd_probe_gather does the same for the second phase: the rate at which wavefronts gather row segments from a
// table, as a function of how many distinct segments there are (which cache level serves them).
#include "lcrwmd_internal.h"

namespace lcrwmd {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// in[i]: random bf16 pairs in +-[0.5, 1) (a hash of i), or zeros
__global__ void k_probe_fill(uint32_t* in, int n, int random)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t x = (uint32_t)i * 2654435761u;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    const uint32_t lo = 0x3F00u + (x & 0xFFu), hi = 0xBF00u + ((x >> 8) & 0xFFu);
    in[i] = random ? (lo | (hi << 16)) : 0u;
}

template <bool BF16, bool A_FROM_LDS>
__global__ __launch_bounds__(256) void k_probe_mfma(const f32x4* __restrict__ in, float* __restrict__ out, int iters,
                                                    long long* __restrict__ clk)
{
    __shared__ f32x4 lds[8 * 256];
    f32x16 acc[4];
    for (int t = 0; t < 4; ++t)
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    f32x4 a[8], b[8];
    for (int i = 0; i < 8; ++i) {
        a[i] = in[(threadIdx.x * 16 + i) % 4096];
        b[i] = in[(threadIdx.x * 16 + 8 + i) % 4096];
        lds[i * 256 + threadIdx.x] = a[i];
    }
    __syncthreads();
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (A_FROM_LDS && (u & 1) == 0) {          // one 16-byte LDS read per lane per two MFMAs
                a[u & 7] = lds[((u + i) & 7) * 256 + threadIdx.x];
                a[(u + 1) & 7] = a[u & 7];
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (BF16)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[(u + t) & 7]),
                                                                    __builtin_bit_cast(bf16x8, b[(u * 3 + t) & 7]), acc[t], 0, 0, 0);
                else
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[(u + t) & 7][t], b[(u * 3 + t) & 7][t], acc[t], 0, 0, 0);
            }
        }
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float s = 0;
    for (int t = 0; t < 4; ++t)
        for (int r = 0; r < 16; ++r) s += acc[t][r];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (threadIdx.x == 0 && blockIdx.x == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
}

// Gathers as the second phase issues them: a wavefront reads the first 64 * W floats (W = 4: 1 KiB, one 16-byte load per
// lane) of a pseudo-random row of a table with a pitch of 16 KiB, eight rows requested before the first is used.  What
// varies is the number of distinct rows, i.e. whether the gathered segments fit an XCD's L2, the Infinity Cache, or
// neither.  Row numbers come from a per-wavefront linear congruential sequence masked to the table's (power of two)
// row count.
template <int W>
__global__ __launch_bounds__(256) void k_probe_gather(const float* __restrict__ T, uint32_t row_mask, int iters, float* __restrict__ out)
{
    typedef float vecw __attribute__((ext_vector_type(W)));
    const int lane = threadIdx.x & 63;
    uint32_t seed = __builtin_amdgcn_readfirstlane((blockIdx.x * 4 + (threadIdx.x >> 6)) * 2654435761u + 12345u);
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        vecw z[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            seed = seed * 1664525u + 1013904223u;
            const uint32_t r = (seed >> 8) & row_mask;
            z[k] = *reinterpret_cast<const vecw*>(T + (int64_t)r * 4096 + lane * W);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k)
#pragma unroll
            for (int t = 0; t < W; ++t) acc += reinterpret_cast<const float*>(&z[k])[t];
    }
    if (acc == 123.456f) out[0] = acc;          // keeps the loads alive; the table holds zeros
}

}  // namespace

// One launch: `blocks` workgroups of four wavefronts, each wavefront `iters` groups of eight gathers of 64 * W floats
// from a table of `rows` rows (a power of two) x 4096 floats at T.  *bytes: what the lanes loaded.
hipError_t launch_probe_gather(const float* T, int64_t rows, int width, int blocks, int iters, float* out, double* bytes,
                               hipStream_t s)
{
    const uint32_t mask = (uint32_t)(rows - 1);
    if (width == 4) k_probe_gather<4><<<blocks, 256, 0, s>>>(T, mask, iters, out);
    else if (width == 2) k_probe_gather<2><<<blocks, 256, 0, s>>>(T, mask, iters, out);
    else k_probe_gather<1><<<blocks, 256, 0, s>>>(T, mask, iters, out);
    *bytes = (double)blocks * 4 * (double)iters * 8 * 64 * width * 4;
    return hipGetLastError();
}

size_t probe_bytes(int num_cu) { return 4096 * 16 + (size_t)num_cu * 2 * 256 * 4 + 256 + 64; }

// One launch of `iters` iterations (32 MFMAs per wavefront each) on 2 workgroups per CU; flops and cycle counts back.
hipError_t launch_probe_mfma(bool bf16, bool random, bool a_from_lds, int iters, int num_cu, void* ws, double* flops,
                             long long** clk_dev, hipStream_t s)
{
    char* base = (char*)ws;
    uint32_t* in = (uint32_t*)base;
    float* out = (float*)(base + 4096 * 16);
    long long* clk = (long long*)(base + 4096 * 16 + (((size_t)num_cu * 2 * 256 * 4 + 255) & ~(size_t)255));
    k_probe_fill<<<64, 256, 0, s>>>(in, 4096 * 4, random ? 1 : 0);
    const int grid = num_cu * 2;
    const f32x4* inp = (const f32x4*)in;
    if (bf16) {
        if (a_from_lds) k_probe_mfma<true, true><<<grid, 256, 0, s>>>(inp, out, iters, clk);
        else k_probe_mfma<true, false><<<grid, 256, 0, s>>>(inp, out, iters, clk);
    } else {
        if (a_from_lds) k_probe_mfma<false, true><<<grid, 256, 0, s>>>(inp, out, iters, clk);
        else k_probe_mfma<false, false><<<grid, 256, 0, s>>>(inp, out, iters, clk);
    }
    *flops = (double)grid * 4 * (double)iters * 32.0 * 2 * 32 * 32 * (bf16 ? 16 : 2);
    *clk_dev = clk;
    return hipGetLastError();
}

}  // namespace lcrwmd
