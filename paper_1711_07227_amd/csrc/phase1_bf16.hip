// Operand packing for the bf16-in / fp32-accumulate first phase of LC-RWMD (Sec. IV, Fig. 6); the contraction
// itself is the tile kernel in phase1_tiles.hip.
//
// Packed operand (pack kernel below): one row per word, 320 bf16 values (five 128-byte lines): columns [0, m)
// hold the embedding rounded to bf16 (round-to-nearest-even), then zeros, and columns 300..302 hold -|row|^2/2
// split into three bf16 terms.  A word used as a TOKEN brings these along; for a word used as VOCABULARY the kernel
// overwrites the same three positions of its register copy with 1.0, so the contraction itself adds the
// -|T_a|^2/2 term and the epilogue is a plain maximum.
//
#include "lcrwmd_internal.h"

namespace lcrwmd {

namespace {

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

// Split copy for the three-product form: value x -> hi = bf16(x), lo = bf16(x - hi); a row holds the 304 hi values
// (zeros beyond m), then the 304 lo values, then zeros up to 640.  The norms are those of the fp32 values.
__global__ __launch_bounds__(256) void k_pack_x3(const float* __restrict__ E, int64_t v, int32_t m, int64_t ld,
                                                 uint16_t* __restrict__ packed, float* __restrict__ normE)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= v) return;
    uint16_t* out = packed + w * 640;
    float s = 0.f;
    for (int t = lane; t < 320; t += 64) {
        uint16_t hi = 0, lo = 0;
        if (t < m) {
            const float x = E[w * ld + t];
            hi = f32_to_bf16_rne(x);
            lo = f32_to_bf16_rne(x - bf16_to_f32(hi));
            s = fmaf(x, x, s);
        }
        if (t < 304) { out[t] = hi; out[304 + t] = lo; }
        else out[304 + t] = 0;            // columns 608 .. 623
    }
    if (lane < 16) out[624 + lane] = 0;
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) normE[w] = s;
}

}  // namespace

// The packed row always has the tile kernel's shape: 320 columns, values in [0, m), zeros up to column 300, the three
// norm terms in columns 300..302 (the last K step's upper half, elements 4..6).
constexpr int32_t kPackPitch = 320, kNormCol = 300;
bool bf16_supported(int32_t m) { return m <= kNormCol; }
int32_t bf16_pitch(int32_t) { return kPackPitch; }
size_t pack_bf16_bytes(int64_t v, int32_t) { return (size_t)v * kPackPitch * 2; }

hipError_t launch_pack_bf16(const void* E, lcrwmd_dtype dtype, int64_t v, int32_t m, int64_t ld, void* packed,
                            float* normE, hipStream_t s)
{
    if (v <= 0) return hipSuccess;
    if (!bf16_supported(m)) return hipErrorNotSupported;
    k_pack_bf16<<<(unsigned)((v + 3) / 4), 256, 0, s>>>(E, dtype == LCRWMD_BF16 ? 1 : 0, v, m, ld, kPackPitch, kNormCol,
                                                       (uint16_t*)packed, normE);
    return hipGetLastError();
}

size_t pack_x3_bytes(int64_t v) { return (size_t)v * 640 * 2; }
int32_t x3_pitch() { return 640; }

hipError_t launch_pack_x3(const float* E, int64_t v, int32_t m, int64_t ld, void* packed, float* normE, hipStream_t s)
{
    if (v <= 0) return hipSuccess;
    if (m > kNormCol) return hipErrorNotSupported;
    k_pack_x3<<<(unsigned)((v + 3) / 4), 256, 0, s>>>(E, v, m, ld, (uint16_t*)packed, normE);
    return hipGetLastError();
}

hipError_t launch_phase1_bf16(const Phase1Args& a, const TokenPlan& tp, hipStream_t s)
{
    if (a.nvoc <= 0 || tp.nseg <= 0) return hipSuccess;
    if (!bf16_supported(a.m)) return hipErrorNotSupported;
    return launch_phase1_tiles_bf16(a, tp, a.num_cu, s);
}

}  // namespace lcrwmd
