// Exact Word Mover's Distance for lists of histogram pairs, the Word Centroid Distance, and the device side of
// RWMD-based pruning (Sec. II: EMD as a transport problem; Sec. III: "Solving the WMD problem", "Speeding-up WMD
// using RWMD", "Word Centroid Distance").
//
// The transport problems are small (tens to hundreds of words a side) and there are many of them, so each is given
// to one wavefront, which forms the pair's cost matrix (fp32) and then runs successive shortest paths with node
// potentials on the dense bipartite graph; everything the solver itself computes (potentials, path lengths, flows,
// the objective) is fp64.  Every loop is bounded by the problem's dimensions, so every wavefront ends.
#include <float.h>
#include <limits.h>

#include <type_traits>

#include "lcrwmd_internal.h"

namespace lcrwmd {

namespace {

constexpr double kFar = 1e300;        // "no path yet"
constexpr double kMassEps = 1e-13;    // mass below this is rounding residue of the fp64 normalisation

__device__ inline float emb_val(const void* E, int dtype, int64_t idx)
{
    if (dtype == LCRWMD_BF16) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(E)[idx] << 16);
    return reinterpret_cast<const float*>(E)[idx];
}

// Order this wavefront's earlier LDS and global accesses before its later ones (lanes hand values to one another).
__device__ inline void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// A value that is the same in every lane, moved to a scalar register.  The solver's control flow depends only on
// such values; saying so keeps its branches scalar, so that every cross-lane operation runs with all lanes active
// (left to itself the compiler treats them as divergent and may route lanes through a loop header separately).
__device__ inline int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Minimum of x over the wavefront, the same value in every lane.  Data-parallel-primitive moves inside rows of 16
// lanes (shifts by 1, 2, 4, 8: lane 15 of a row ends up with the row's minimum), then row 0 -> row 1 and row 2 -> row 3,
// then rows 0-1 -> rows 2-3; lane 63 holds the result.  A lane without a source keeps its own value.
template <int CTRL, int ROW_MASK>
__device__ inline double dpp_min_step(double x)
{
    const int lo = __double2loint(x), hi = __double2hiint(x);
    const int olo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, ROW_MASK, 0xf, false);
    const int ohi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, ROW_MASK, 0xf, false);
    const double o = __hiloint2double(ohi, olo);
    return o < x ? o : x;
}

__device__ inline double wave_min(double x)
{
    x = dpp_min_step<0x111, 0xf>(x);      // row_shr:1
    x = dpp_min_step<0x112, 0xf>(x);      // row_shr:2
    x = dpp_min_step<0x114, 0xf>(x);      // row_shr:4
    x = dpp_min_step<0x118, 0xf>(x);      // row_shr:8
    x = dpp_min_step<0x142, 0xa>(x);      // row_bcast:15 into rows 1 and 3
    x = dpp_min_step<0x143, 0xc>(x);      // row_bcast:31 into rows 2 and 3
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), 63), hi = __builtin_amdgcn_readlane(__double2hiint(x), 63);
    return __hiloint2double(hi, lo);
}

// the same for a float, one instruction per step
template <int CTRL, int ROW_MASK>
__device__ inline float dpp_min_step(float x)
{
    const int o = __builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
    return fminf(x, __int_as_float(o));
}

__device__ inline float wave_min(float x)
{
    x = dpp_min_step<0x111, 0xf>(x);
    x = dpp_min_step<0x112, 0xf>(x);
    x = dpp_min_step<0x114, 0xf>(x);
    x = dpp_min_step<0x118, 0xf>(x);
    x = dpp_min_step<0x142, 0xa>(x);
    x = dpp_min_step<0x143, 0xc>(x);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

__device__ inline double wave_sum(double x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// ---------------------------------------------------------------------------------------------------------------
// C = T1 o T2 of one pair (Sec. III), by one wavefront: c[p * h2 + u] = || E[word p of X1[i]] - E[word u of X2[j]] ||.
//
// 32 x 32 output tiles, the embedding dimension staged through LDS 16 values at a time.  A tile is first evaluated on
// the matrix cores as |a|^2 + |b|^2 - 2 a.b (v_mfma_f32_32x32x2_f32, fp32 throughout; the norms are summed from the
// very operand values the products use).  That form loses digits where two different words lie close together, so a
// tile holding any entry with d^2 < kCloseFrac (|a|^2 + |b|^2) is evaluated again from coordinate differences, and
// equal word ids give exactly 0 either way.  What is kept from the expansion therefore has a relative error of the
// order of the fp32 dot product's own (m roundings, about 1e-6) divided by 2 kCloseFrac.
// `tiles` is cost_lds_bytes(slice width) bytes of this wavefront's LDS.
// ---------------------------------------------------------------------------------------------------------------
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kCT = 32;      // tile edge
constexpr float kCloseFrac = 0.25f;
// LDS of the tile buffers for slices of CK embedding values: two 32-row operand tiles, word ids, norms
constexpr int cost_lds_bytes(int CK) { return (2 * kCT * (CK + 1) + 4 * kCT) * 4; }

// What a lane gathers of one slice (CK embedding values of the tile's 32 + 32 rows), and how.
//   VEC: CK / 4 lanes per row, each one group of four values as one 16-byte (fp32) or 8-byte (bf16) load, so that a
//        row's share of the slice is one contiguous request of 4 CK bytes (a whole 128-byte line for CK = 32); needs
//        the rows to start on such boundaries (base address and pitch), which the caller checks.
//   else: CK lanes per row, one element per load.
template <typename TE>
struct Vec4;
template <>
struct Vec4<float> { typedef float4 type; };
template <>
struct Vec4<uint16_t> { typedef uint2 type; };

template <typename TE, bool VEC, int CK>
struct Gather;
template <typename TE, int CK>
struct Gather<TE, true, CK> { typename Vec4<TE>::type a[CK / 8], b[CK / 8]; };
template <typename TE, int CK>
struct Gather<TE, false, CK> { TE a[CK / 2], b[CK / 2]; };

__device__ inline float as_float(float x) { return x; }
__device__ inline float as_float(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }      // bf16 bits
__device__ inline void unpack4(const float4& v, float (&f)[4]) { f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w; }
__device__ inline void unpack4(const uint2& v, float (&f)[4])
{
    f[0] = __uint_as_float(v.x << 16);
    f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16);
    f[3] = __uint_as_float(v.y & 0xffff0000u);
}

template <int CK>
struct CostTile {
    float (*A)[CK + 1];
    float (*B)[CK + 1];
    int32_t* wa;
    int32_t* wb;
    float* nA;
    __device__ explicit CostTile(float* tiles)
        : A(reinterpret_cast<float (*)[CK + 1]>(tiles)), B(reinterpret_cast<float (*)[CK + 1]>(tiles + kCT * (CK + 1))),
          wa(reinterpret_cast<int32_t*>(tiles + 2 * kCT * (CK + 1))), wb(wa + kCT),
          nA(tiles + 2 * kCT * (CK + 1) + 2 * kCT)
    {
    }
    // word ids of the tile's rows and columns; past the end of a histogram its last word again (never stored)
    __device__ void set_words(const int32_t* __restrict__ wa_g, int p0, int h1, const int32_t* __restrict__ wb_g, int u0, int h2,
                              int lane) const
    {
        if (lane < kCT) wa[lane] = wa_g[p0 + lane < h1 ? p0 + lane : h1 - 1];
        else wb[lane - kCT] = wb_g[u0 + lane - kCT < h2 ? u0 + lane - kCT : h2 - 1];
    }
    // Slice k0: `fetch` requests a lane's share (all loads in flight together), `put` writes it to A and B with zeros
    // past m.  Word ids and pitches are below 2^31: one 32 x 32 -> 64 bit multiply per row.
    template <typename TE>
    __device__ void fetch(const TE* __restrict__ E, int64_t ld, int32_t m, int k0, int lane, Gather<TE, false, CK>& g) const
    {
        constexpr int RP = 64 / CK;                   // rows per pass
        const int lr = lane / CK, lc = lane % CK;
        const uint32_t kk = k0 + lc < m ? k0 + lc : m - 1;
        const uint32_t pitch = (uint32_t)ld;
#pragma unroll
        for (int e = 0; e < CK / 2; ++e) {
            g.a[e] = E[(uint64_t)(uint32_t)wa[lr + RP * e] * pitch + kk];
            g.b[e] = E[(uint64_t)(uint32_t)wb[lr + RP * e] * pitch + kk];
        }
    }
    template <typename TE>
    __device__ void put(int32_t m, int k0, int lane, const Gather<TE, false, CK>& g) const
    {
        constexpr int RP = 64 / CK;
        const int lr = lane / CK, lc = lane % CK;
        const bool kin = k0 + lc < m;
#pragma unroll
        for (int e = 0; e < CK / 2; ++e) {
            A[lr + RP * e][lc] = kin ? as_float(g.a[e]) : 0.f;
            B[lr + RP * e][lc] = kin ? as_float(g.b[e]) : 0.f;
        }
    }
    // the pitch is a multiple of 4 here, so a group of four values that starts below m ends inside the row's pitch
    template <typename TE>
    __device__ void fetch(const TE* __restrict__ E, int64_t ld, int32_t m, int k0, int lane, Gather<TE, true, CK>& g) const
    {
        constexpr int LR = CK / 4, RP = 64 / LR;      // lanes per row, rows per pass
        const int lr = lane / LR;
        const int k4 = k0 + 4 * (lane % LR);
        const uint32_t kk = k4 < m ? k4 : 0;
        const uint32_t pitch = (uint32_t)ld;
        typedef typename Vec4<TE>::type V;
#pragma unroll
        for (int e = 0; e < CK / 8; ++e) {
            g.a[e] = *reinterpret_cast<const V*>(E + ((uint64_t)(uint32_t)wa[lr + RP * e] * pitch + kk));
            g.b[e] = *reinterpret_cast<const V*>(E + ((uint64_t)(uint32_t)wb[lr + RP * e] * pitch + kk));
        }
    }
    template <typename TE>
    __device__ void put(int32_t m, int k0, int lane, const Gather<TE, true, CK>& g) const
    {
        constexpr int LR = CK / 4, RP = 64 / LR;
        const int lr = lane / LR, lc = 4 * (lane % LR);
#pragma unroll
        for (int e = 0; e < CK / 8; ++e) {
            float fa[4], fb[4];
            unpack4(g.a[e], fa);
            unpack4(g.b[e], fb);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const bool kin = k0 + lc + t < m;
                A[lr + RP * e][lc + t] = kin ? fa[t] : 0.f;
                B[lr + RP * e][lc + t] = kin ? fb[t] : 0.f;
            }
        }
    }
};

// one tile from coordinate differences (no norm expansion): 4 x 4 outputs per lane, rows ty + 8 a, columns tx + 8 b
template <typename TE, bool VEC, int CK>
__device__ __forceinline__ void cost_tile_exact(const CostTile<CK>& T, const TE* __restrict__ E, int64_t ld, int32_t m, int p0,
                                                int h1, int u0, int h2, float* c, int lane)
{
    const int tx = lane & 7, ty = lane >> 3;
    float acc[4][4] = {};
    Gather<TE, VEC, CK> g;
    for (int k0 = 0; k0 < m; k0 += CK) {
        T.fetch(E, ld, m, k0, lane, g);
        wave_sync();                               // the previous slice has been consumed
        T.put(m, k0, lane, g);
        wave_sync();
#pragma unroll 4
        for (int k = 0; k < CK; ++k) {
            float x[4], y[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) { x[e] = T.A[ty + 8 * e][k]; y[e] = T.B[tx + 8 * e][k]; }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const float d = x[a] - y[b];
                    acc[a][b] = fmaf(d, d, acc[a][b]);
                }
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int p = p0 + ty + 8 * a, u = u0 + tx + 8 * b;
            if (p < h1 && u < h2) c[(int64_t)p * h2 + u] = sqrtf(acc[a][b]);
        }
}

template <typename TE, bool VEC, int CK>
__device__ __forceinline__ void pair_costs_as(const TE* __restrict__ E, int64_t ld, int32_t m, const int32_t* __restrict__ wa_g,
                                              int h1, const int32_t* __restrict__ wb_g, int h2, float* c, float* tiles, int lane)
{
    const CostTile<CK> T(tiles);
    const int l31 = lane & 31, half = lane >> 5;
    Gather<TE, VEC, CK> g;
    for (int p0 = 0; p0 < h1; p0 += kCT)
        for (int u0 = 0; u0 < h2; u0 += kCT) {
            wave_sync();                           // the previous tile's ids and norms have been read
            T.set_words(wa_g, p0, h1, wb_g, u0, h2, lane);
            wave_sync();
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
            float na = 0.f, nb = 0.f;
            T.fetch(E, ld, m, 0, lane, g);
            for (int k0 = 0; k0 < m; k0 += CK) {
                wave_sync();                       // the previous slice has been consumed
                T.put(m, k0, lane, g);
                wave_sync();
                if (k0 + CK < m) T.fetch(E, ld, m, k0 + CK, lane, g);             // in flight behind this slice's products
#pragma unroll
                for (int i = 0; i < CK / 2; ++i) {
                    const float a = T.A[l31][2 * i + half], b = T.B[l31][2 * i + half];
                    na = fmaf(a, a, na);
                    nb = fmaf(b, b, nb);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
                }
            }
            na += __shfl_xor(na, 32);              // both halves of the embedding dimension
            nb += __shfl_xor(nb, 32);
            if (half == 0) T.nA[l31] = na;
            wave_sync();
            // accumulator register v of a lane: row 8 (v / 4) + 4 half + v % 4 of the tile, column l31
            const int32_t wcol = T.wb[l31];
            const bool col_in = u0 + l31 < h2;
            bool close = false;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = 8 * (v >> 2) + 4 * half + (v & 3);
                const float s = T.nA[i] + nb;
                close |= col_in && p0 + i < h1 && T.wa[i] != wcol && s - 2.f * acc[v] < kCloseFrac * s;
            }
            if (uni(__any(close) ? 1 : 0)) {
                cost_tile_exact<TE, VEC, CK>(T, E, ld, m, p0, h1, u0, h2, c, lane);
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = 8 * (v >> 2) + 4 * half + (v & 3);
                    if (col_in && p0 + i < h1)
                        c[(int64_t)(p0 + i) * h2 + u0 + l31] =
                            T.wa[i] == wcol ? 0.f : sqrtf(fmaxf(T.nA[i] + nb - 2.f * acc[v], 0.f));
                }
            }
        }
    wave_sync();                                   // the tile buffers become the solver's state
}

// CKV: slice width of the vectorised gathers (`tiles` holds cost_lds_bytes(CKV) bytes)
template <int CKV>
__device__ __forceinline__ void pair_costs(const void* __restrict__ E, int dtype, int64_t ld, int32_t m,
                                           const int32_t* __restrict__ wa_g, int h1, const int32_t* __restrict__ wb_g, int h2,
                                           float* c, float* tiles, int lane)
{
    // groups of four values per load where every row starts on a group's boundary
    const bool bf = dtype == LCRWMD_BF16;
    const bool vec = (ld & 3) == 0 && (reinterpret_cast<uintptr_t>(E) & (bf ? 7 : 15)) == 0;
    if (bf) {
        const uint16_t* Eb = reinterpret_cast<const uint16_t*>(E);
        if (vec) pair_costs_as<uint16_t, true, CKV>(Eb, ld, m, wa_g, h1, wb_g, h2, c, tiles, lane);
        else pair_costs_as<uint16_t, false, 16>(Eb, ld, m, wa_g, h1, wb_g, h2, c, tiles, lane);
    } else {
        const float* Ef = reinterpret_cast<const float*>(E);
        if (vec) pair_costs_as<float, true, CKV>(Ef, ld, m, wa_g, h1, wb_g, h2, c, tiles, lane);
        else pair_costs_as<float, false, 16>(Ef, ld, m, wa_g, h1, wb_g, h2, c, tiles, lane);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// EMD of one pair per wavefront (Sec. II): minimise sum y[p,u] c[p,u] with row sums x1, column sums x2, y >= 0.
//
// Successive shortest paths.  Node potentials phiS (words of X1[i], "sources") and phiT (words of X2[j], "sinks")
// keep every reduced cost c[p,u] + phiS[p] - phiT[u] non-negative and make it zero on edges that carry flow.  The
// sources are served one after the other; while source s has mass left, a Dijkstra search over the residual graph
// finds the nearest sink with unmet demand: forward edges exist between every source and every sink, a backward
// edge from sink u to source p exists where y[p,u] > 0 and has reduced cost zero, so a source enters the search at
// the distance of the sink that reaches it.  Mass min(supply left, demand left, smallest flow on a backward edge
// of the path) is moved and the objective grows by mass x path cost.  If that filled the sink and emptied no
// backward edge, the search goes on from where it stands (the sink now passes flow on like any full sink);
// otherwise it ends, the potentials are shifted by the search distances, and the next search starts.
// Lane l owns sinks and sources l, l + 64, ...; their per-node state sits in LDS, the flow matrix (transposed: one
// row per sink) and the costs in the wavefront's slab in device memory.  Which entries of the flow matrix are
// positive is also kept as one bit each in LDS when that fits (bm_words > 0 words per sink), so that a search reads
// device memory only for rows of the cost matrix.
// Histogram weights are divided by their fp64 sums first, so both sides carry mass 1.
//
// The grid is a set of wavefronts that take pairs off a shared counter until it passes `count`: every wavefront
// ends because every loop below is bounded by the pair's dimensions or by the augmentation budget.
// flags[t]: 0 solved; 1 the augmentation budget ran out (the result is then the cost of a partial flow).
//
// Giving up above a limit (limit != nullptr: pair t only matters if its distance is at most limit[j - limit_j0]).
// Between searches the potentials are a feasible point of the dual programme whose value is the cost of the flow so
// far plus, for every source with supply left, that supply times its dual variable: the negated potential of the
// source being served, and for a source not yet served any r with r <= c[p, u] - phiT[u] for all u, in particular
// r_p = min_u c[p, u] because the potentials of sinks only ever fall.  The value of a dual point bounds the optimum
// from below, so once  total + sup[s] max(r_s, -phiS[s]) + sum_{p > s} x1[p] r_p  exceeds the limit the pair is
// abandoned: out[t] = FLT_MAX, one more in give_up_count.  (At the start the bound is the one-sided RWMD.)
//
// NPL > 0 (histograms of the query side of at most 64 NPL words): the potentials and the tentative distances of a
// lane's sinks live in registers, so that settling a node touches LDS only to record a predecessor; NPL == 0: any
// size, that state in LDS.
// ---------------------------------------------------------------------------------------------------------------
// slices of the cost tiles: 16 values in every variant (32, whole 128-byte lines per row, measured 4 % slower on
// 100-word histograms and would take more LDS than the per-word state of small problems)
constexpr int emd_slice(int) { return 16; }

template <int NPL>
__global__ __launch_bounds__(64, NPL == 2 ? 6 : 4) void k_emd(const void* __restrict__ E, int dtype, int64_t ld, int32_t m,
                                            const int64_t* __restrict__ db_rp, const int32_t* __restrict__ db_col,
                                            const float* __restrict__ db_val, const int64_t* __restrict__ q_rp,
                                            const int32_t* __restrict__ q_col, const float* __restrict__ q_val,
                                            const int32_t* __restrict__ pair_db, const int32_t* __restrict__ pair_q,
                                            int64_t count, int32_t* next_pair, float* slabs_c, int64_t slab_elems,
                                            double* slabs_f, int32_t h1max, int32_t h2max, int32_t bm_words,
                                            float* __restrict__ out,
                                            int32_t* __restrict__ flags, int32_t* fail_count,
                                            const float* __restrict__ limit, int32_t limit_j0, int32_t* give_up_count)
{
    extern __shared__ double lds_d[];
    double* phiS = lds_d;
    double* dS = phiS + h1max;
    double* sup = dS + h1max;
    // the register variants keep the sinks' potentials and tentative distances out of LDS altogether
    constexpr bool REG = NPL > 0;
    double* phiT = sup + h1max;
    double* dT = phiT + (REG ? 0 : h2max);
    double* dem = REG ? sup + h1max : dT + h2max;
    int32_t* par = reinterpret_cast<int32_t*>(dem + h2max);
    int32_t* way = par + h1max;
    uint32_t* bm = reinterpret_cast<uint32_t*>(way + h2max);        // [h2max][bm_words], bit p of row u: y[p, u] > 0

    constexpr int NR = REG ? NPL : 1;
    const int lane = threadIdx.x;
    float* c = slabs_c + (int64_t)blockIdx.x * slab_elems;
    double* f = slabs_f + (int64_t)blockIdx.x * slab_elems;          // f[u * h1 + p] = y[p, u]
    double pT[NR], dTr[NR];                                          // REG: potential / distance of sink lane + 64 k

    for (;;) {
        wave_sync();                                                 // the previous pair's state has been read
        int32_t got = 0;
        if (lane == 0) got = atomicAdd(next_pair, 1);
        const int32_t t = uni(got);
        if (t >= count) break;
        const int32_t i = pair_db[t], j = pair_q[t];
        const int64_t a0 = db_rp[i], b0 = q_rp[j];
        const int h1 = uni((int)(db_rp[i + 1] - a0)), h2 = uni((int)(q_rp[j + 1] - b0));

        double sa = 0.0, sb = 0.0;
        for (int p = lane; p < h1; p += 64) sa += (double)db_val[a0 + p];
        for (int u = lane; u < h2; u += 64) sb += (double)q_val[b0 + u];
        sa = wave_sum(sa);
        sb = wave_sum(sb);

        pair_costs<emd_slice(NPL)>(E, dtype, ld, m, db_col + a0, h1, q_col + b0, h2, c, reinterpret_cast<float*>(lds_d), lane);
        for (int p = lane; p < h1; p += 64) { phiS[p] = 0.0; sup[p] = (double)db_val[a0 + p] / sa; }
        for (int u = lane; u < h2; u += 64) {
            if constexpr (!REG) phiT[u] = 0.0;
            dem[u] = (double)q_val[b0 + u] / sb;
        }
#pragma unroll
        for (int k = 0; k < NR; ++k) pT[k] = 0.0;
        // with the map of positive flows an entry of f is read only after it has been written: no need to clear f
        if (!bm_words)
            for (int64_t e = lane; e < (int64_t)h1 * h2; e += 64) f[e] = 0.0;
        for (int e = lane; e < h2 * bm_words; e += 64) bm[e] = 0u;
        wave_sync();

        const int budget = 8 * (h1 + h2) + 64;     // augmentations; each empties a source, a sink or a flow entry
        int naug = 0;
        bool exhausted = false, abandoned = false;
        double total = 0.0;

        // what the sources not yet served must at least pay: sum of x1[p] min_u c[p, u]
        const bool bounded = limit != nullptr;
        const double lim = bounded ? (double)limit[j - limit_j0] : 0.0;
        double tail = 0.0;
        if (bounded) {
            for (int p = 0; p < h1; ++p) {                       // rows read whole, lanes over the sinks
                const float* row = c + (int64_t)p * h2;
                float r = FLT_MAX;
                for (int u = lane; u < h2; u += 64) r = fminf(r, row[u]);
                r = wave_min(r);
                if (lane == (p & 63)) tail += sup[p] * (double)r;
            }
            tail = wave_sum(tail);
        }

        for (int s = 0; s < h1 && !exhausted && !abandoned; ++s) {
            double r_s = 0.0, paid = 0.0;           // bounded: min_u c[s, u]; sum of this source's search distances
            if (bounded) {
                const float* row = c + (int64_t)s * h2;
                float r = FLT_MAX;
                for (int u = lane; u < h2; u += 64) r = fminf(r, row[u]);
                r_s = (double)wave_min(r);
                tail -= sup[s] * r_s;
                tail = tail > 0.0 ? tail : 0.0;
            }
            while (uni(sup[s] > kMassEps)) {
                if (naug >= budget) { exhausted = true; break; }
                // ---- search from s ----
                // bit r of a lane's masks: its sink / source lane + 64 r has been settled by this search
                uint32_t used = 0, vis = 0;
                wave_sync();
                if (lane == (s & 63)) { vis = 1u << (s >> 6); dS[s] = 0.0; par[s] = -1; }
                {
                    const double ps = phiS[s];
                    const float* crow = c + (int64_t)s * h2;
                    if constexpr (REG) {
#pragma unroll
                        for (int k = 0; k < NR; ++k) {
                            const int u = lane + 64 * k;
                            dTr[k] = kFar;
                            if (u < h2) {
                                const double rc = (double)crow[u] + ps - pT[k];
                                dTr[k] = rc > 0.0 ? rc : 0.0;
                                way[u] = s;
                            }
                        }
                    } else {
                        for (int u = lane; u < h2; u += 64) {
                            double rc = (double)crow[u] + ps - phiT[u];
                            dT[u] = rc > 0.0 ? rc : 0.0;
                            way[u] = s;
                        }
                    }
                }
                bool reached = false;
                double Dt = 0.0;
                for (int it = 0; it < h2; ++it) {
                    double bv = kFar;
                    int bi = INT_MAX;
                    if constexpr (REG) {
#pragma unroll
                        for (int k = 0; k < NR; ++k)                // sinks past the end carry kFar
                            if (!((used >> k) & 1) && dTr[k] < bv) { bv = dTr[k]; bi = lane + 64 * k; }
                    } else {
                        for (int u = lane, r = 0; u < h2; u += 64, ++r)
                            if (!((used >> r) & 1) && dT[u] < bv) { bv = dT[u]; bi = u; }
                    }
                    // the nearest over all lanes; of equally near sinks the one in the lowest lane
                    const double nearest = wave_min(bv);
                    const unsigned long long holders = __ballot(bi != INT_MAX && bv == nearest);
                    if (holders == 0ull) break;                    // every sink has been taken
                    const int u = __builtin_amdgcn_readlane(bi, __ffsll((long long)holders) - 1);
                    bv = nearest;
                    if (lane == (u & 63)) used |= 1u << (u >> 6);
                    if (uni(dem[u] > 0.0)) {
                        // ---- a sink with unmet demand at distance bv: walk the path back to s for the amount ----
                        reached = true;
                        Dt = bv;
                        wave_sync();                                 // dS / par of sources added since the last sync
                        double delta = sup[s] < dem[u] ? sup[s] : dem[u];
                        {
                            int p = uni(way[u]);
                            for (int g = 0; g < h1; ++g) {
                                const int up = uni(par[p]);
                                if (up < 0) break;
                                const double fl = f[(int64_t)up * h1 + p];
                                delta = fl < delta ? fl : delta;
                                p = uni(way[up]);
                            }
                        }
                        // potentials are those of the search's start; REG: sink u's sits in register u / 64 of lane u % 64
                        double phiT_u;
                        if constexpr (REG) {
                            double mine = pT[0];
#pragma unroll
                            for (int k = 1; k < NR; ++k) mine = (u >> 6) == k ? pT[k] : mine;
                            phiT_u = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(mine), u & 63),
                                                      __builtin_amdgcn_readlane(__double2loint(mine), u & 63));
                        } else {
                            phiT_u = phiT[u];
                        }
                        total += delta * (bv - phiS[s] + phiT_u);
                        wave_sync();                                 // reads of the old flows are done
                        int cut = 0;
                        if (lane == 0) {                             // move the mass
                            int uu = u, p = way[uu];
                            for (int g = 0; g <= h1; ++g) {
                                if (bm_words) {
                                    const uint32_t w = bm[uu * bm_words + (p >> 5)], bit = 1u << (p & 31);
                                    f[(int64_t)uu * h1 + p] = (w & bit) ? f[(int64_t)uu * h1 + p] + delta : delta;
                                    bm[uu * bm_words + (p >> 5)] = w | bit;
                                } else {
                                    f[(int64_t)uu * h1 + p] += delta;
                                }
                                const int up = par[p];
                                if (up < 0) break;
                                const double nf = f[(int64_t)up * h1 + p] - delta;
                                if (nf > kMassEps) f[(int64_t)up * h1 + p] = nf;
                                else {
                                    f[(int64_t)up * h1 + p] = 0.0;
                                    if (bm_words) bm[up * bm_words + (p >> 5)] &= ~(1u << (p & 31));
                                    cut = 1;
                                }
                                uu = up;
                                p = way[uu];
                            }
                            double r = sup[s] - delta;
                            sup[s] = r > kMassEps ? r : 0.0;
                            r = dem[u] - delta;
                            dem[u] = r > kMassEps ? r : 0.0;
                        }
                        cut = uni(cut);
                        wave_sync();
                        ++naug;
                        // go on only if the sink is full now, s has mass left and no backward edge emptied
                        if (cut || naug >= budget || uni(sup[s] <= kMassEps || dem[u] > 0.0)) break;
                    }
                    // sources that send flow to u join the search at u's distance
                    const double* frow = f + (int64_t)u * h1;
                    for (int pb = 0; pb < h1; pb += 64) {
                        const int p = pb + lane;
                        bool add = p < h1 && !((vis >> (pb >> 6)) & 1);
                        if (add) add = bm_words ? ((bm[u * bm_words + (p >> 5)] >> (p & 31)) & 1u) != 0u : frow[p] > 0.0;
                        if (add) { vis |= 1u << (pb >> 6); dS[p] = bv; par[p] = u; }
                        unsigned long long mask = __ballot(add);
                        while (mask) {
                            const int pp = pb + __ffsll((long long)mask) - 1;
                            mask &= mask - 1;
                            const double ps = phiS[pp];
                            const float* crow = c + (int64_t)pp * h2;
                            if constexpr (REG) {
#pragma unroll
                                for (int k = 0; k < NR; ++k) {
                                    const int uu = lane + 64 * k;
                                    if (uu < h2 && !((used >> k) & 1)) {
                                        double rc = (double)crow[uu] + ps - pT[k];
                                        rc = rc > 0.0 ? rc : 0.0;
                                        const double nd = bv + rc;
                                        if (nd < dTr[k]) { dTr[k] = nd; way[uu] = pp; }
                                    }
                                }
                            } else {
                                for (int uu = lane, r = 0; uu < h2; uu += 64, ++r)
                                    if (!((used >> r) & 1)) {
                                        double rc = (double)crow[uu] + ps - phiT[uu];
                                        rc = rc > 0.0 ? rc : 0.0;
                                        const double nd = bv + rc;
                                        if (nd < dT[uu]) { dT[uu] = nd; way[uu] = pp; }
                                    }
                            }
                        }
                    }
                }
                wave_sync();
                if (!reached) {                                     // only rounding residue is left on this side
                    if (lane == (s & 63)) sup[s] = 0.0;
                    wave_sync();
                    break;
                }
                // ---- potentials: nodes the search settled move by their distance minus the last target's ----
                // (a search that went on past its last target may have settled nodes farther away: those stay)
                for (int p = lane, r = 0; p < h1; p += 64, ++r)
                    if (((vis >> r) & 1) && dS[p] < Dt) phiS[p] += dS[p] - Dt;
                if constexpr (REG) {
#pragma unroll
                    for (int k = 0; k < NR; ++k)
                        if (((used >> k) & 1) && dTr[k] < Dt) pT[k] += dTr[k] - Dt;
                } else {
                    for (int u = lane, r = 0; u < h2; u += 64, ++r)
                        if (((used >> r) & 1) && dT[u] < Dt) phiT[u] += dT[u] - Dt;
                }
                wave_sync();
                if (bounded) {
                    paid += Dt;                                    // -phiS[s]
                    const double bound = total + sup[s] * (paid > r_s ? paid : r_s) + tail;
                    if (uni(bound * (1.0 - 1e-9) > lim)) { abandoned = true; break; }
                }
            }
        }
        if (lane == 0) {
            out[t] = abandoned ? FLT_MAX : (float)total;
            if (flags) flags[t] = exhausted ? 1 : 0;
            if (exhausted && fail_count) atomicAdd(fail_count, 1);
            if (abandoned && give_up_count) atomicAdd(give_up_count, 1);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Word Centroid Distance (Sec. III): centroids X E, then Euclidean distances between centroids.
// ---------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_centroids(const void* __restrict__ E, int dtype, int64_t ld, int32_t m,
                                                   const int64_t* __restrict__ rp, const int32_t* __restrict__ col,
                                                   const float* __restrict__ val, float* __restrict__ C, int64_t ldc)
{
    const int64_t i = blockIdx.x;
    const int64_t a = rp[i], b = rp[i + 1];
    for (int k = threadIdx.x; k < m; k += 256) {
        float acc = 0.f;
        for (int64_t e = a; e < b; ++e) acc = fmaf(val[e], emb_val(E, dtype, (int64_t)col[e] * ld + k), acc);
        C[i * ldc + k] = acc;
    }
}

// D[i * ldd + j] = || C1[i] - C2[j] ||: 64 x 64 outputs per workgroup, 4 x 4 per thread, 16 dimensions per LDS slice.
__global__ __launch_bounds__(256) void k_centroid_dist(const float* __restrict__ C1, int64_t n, const float* __restrict__ C2,
                                                       int64_t q, int64_t ldc, int32_t m, float* __restrict__ D, int64_t ldd)
{
    __shared__ float A[16][64 + 1], B[16][64 + 1];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t i0 = (int64_t)blockIdx.y * 64, j0 = (int64_t)blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < m; k0 += 16) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int r = (tid >> 4) + 16 * e, k = tid & 15;
            A[k][r] = (i0 + r < n && k0 + k < m) ? C1[(i0 + r) * ldc + k0 + k] : 0.f;
            B[k][r] = (j0 + r < q && k0 + k < m) ? C2[(j0 + r) * ldc + k0 + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float x[4], y[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) { x[e] = A[k][ty + 16 * e]; y[e] = B[k][tx + 16 * e]; }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const float d = x[a] - y[b];
                    acc[a][b] = fmaf(d, d, acc[a][b]);
                }
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int64_t i = i0 + ty + 16 * a, j = j0 + tx + 16 * b;
            if (i < n && j < q) D[i * ldd + j] = sqrtf(acc[a][b]);
        }
}

// ---------------------------------------------------------------------------------------------------------------
// Pruning (Sec. III, "Speeding-up WMD using RWMD").  D is the n x q tile of RWMD bounds, R0 the k nearest by RWMD.
// ---------------------------------------------------------------------------------------------------------------
// pair lists of candidates lo .. hi - 1 of every query (R0 holds `stride` of them per query, nearest first), and those
// entries of D masked so that they are not chosen again
__global__ void k_first_pairs(const int32_t* __restrict__ R0, int64_t q, int stride, int lo, int hi, int32_t j0,
                              float* __restrict__ D, int64_t ldd, int32_t* __restrict__ pair_db, int32_t* __restrict__ pair_q)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int w = hi - lo;
    if (e >= q * w) return;
    const int64_t j = e / w;
    const int32_t i = R0[j * stride + lo + (int)(e - j * w)];
    pair_db[e] = i;
    pair_q[e] = j0 + (int32_t)j;
    D[(int64_t)i * ldd + j] = FLT_MAX;
}

// cut[j] = (k-th smallest WMD among the ka + kb >= k evaluated so far: ka per query in wa, kb in wb) * (1 + slack);
// with ka == k and kb == 0 their largest.  At least k of them are finite (abandoned ones hold FLT_MAX).
__global__ void k_cutoff(const float* __restrict__ wa, int ka, const float* __restrict__ wb, int kb, int64_t q, int k,
                         float slack, float* __restrict__ cut)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= q) return;
    const int k1 = ka + kb;
    // k rounds of "smallest value after the last one taken", equal values told apart by position
    float last = -1.f;
    int last_r = -1;
    for (int t = 0; t < k; ++t) {
        float best = FLT_MAX;
        int best_r = k1;
        for (int r = 0; r < k1; ++r) {
            const float x = r < ka ? wa[j * ka + r] : wb[j * kb + r - ka];
            const bool after = x > last || (x == last && r > last_r);
            if (after && (x < best || (x == best && r < best_r))) { best = x; best_r = r; }
        }
        last = best;
        last_r = best_r;
    }
    cut[j] = last * (1.f + slack);
}

constexpr int kRowsPerBlock = 256;

// cnt[j] += rows of this block with D[i][j] < cut[j]      (thread = query column, so reads of D are contiguous)
__global__ __launch_bounds__(256) void k_count_below(const float* __restrict__ D, int64_t n, int64_t q, int64_t ldd,
                                                     const float* __restrict__ cut, int32_t* __restrict__ cnt)
{
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= q) return;
    const int64_t i0 = (int64_t)blockIdx.y * kRowsPerBlock;
    const int64_t i1 = i0 + kRowsPerBlock < n ? i0 + kRowsPerBlock : n;
    const float L = cut[j];
    int32_t c = 0;
    for (int64_t i = i0; i < i1; ++i) c += D[i * ldd + j] < L ? 1 : 0;
    if (c) atomicAdd(&cnt[j], c);
}

// exclusive prefix sums of cnt[0..q) into off[0..q]; one workgroup
__global__ __launch_bounds__(1024) void k_scan_counts(const int32_t* __restrict__ cnt, int64_t q, int64_t* __restrict__ off)
{
    __shared__ int64_t part[1024];
    const int tid = threadIdx.x;
    const int64_t per = (q + 1023) / 1024;
    const int64_t a = tid * per, b = a + per < q ? a + per : q;
    int64_t sum = 0;
    for (int64_t j = a; j < b; ++j) sum += cnt[j];
    part[tid] = sum;
    __syncthreads();
    if (tid == 0) {
        int64_t run = 0;
        for (int k = 0; k < 1024; ++k) { const int64_t x = part[k]; part[k] = run; run += x; }
        off[q] = run;
    }
    __syncthreads();
    int64_t run = part[tid];
    for (int64_t j = a; j < b; ++j) { off[j] = run; run += cnt[j]; }
}

// cursor[j] = start of query j's list relative to the first query of the range
__global__ void k_init_cursor(const int64_t* __restrict__ off, int64_t ja, int64_t jb, int64_t* __restrict__ cursor)
{
    const int64_t j = ja + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < jb) cursor[j] = off[j] - off[ja];
}

// second sweep with the same geometry over the query columns [ja, jb): every thread reserves room for its rows in
// its query's list and fills it
__global__ __launch_bounds__(256) void k_fill_below(const float* __restrict__ D, int64_t n, int64_t ja, int64_t jb,
                                                    int64_t ldd, const float* __restrict__ cut, int64_t* __restrict__ cursor,
                                                    int32_t j0, int32_t* __restrict__ pair_db, int32_t* __restrict__ pair_q)
{
    const int64_t j = ja + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= jb) return;
    const int64_t i0 = (int64_t)blockIdx.y * kRowsPerBlock;
    const int64_t i1 = i0 + kRowsPerBlock < n ? i0 + kRowsPerBlock : n;
    const float L = cut[j];
    int32_t c = 0;
    for (int64_t i = i0; i < i1; ++i) c += D[i * ldd + j] < L ? 1 : 0;
    if (!c) return;
    int64_t at = (int64_t)atomicAdd(reinterpret_cast<unsigned long long*>(&cursor[j]), (unsigned long long)c);
    for (int64_t i = i0; i < i1; ++i)
        if (D[i * ldd + j] < L) { pair_db[at] = (int32_t)i; pair_q[at] = j0 + (int32_t)j; ++at; }
}

__global__ void k_check_pairs(const int32_t* __restrict__ pair_db, const int32_t* __restrict__ pair_q, int64_t npairs,
                              int64_t n, int64_t q, int32_t* __restrict__ status)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= npairs) return;
    const int32_t i = pair_db[t], j = pair_q[t];
    if (i < 0 || i >= n || j < 0 || j >= q) status[0] = 1;
}

// The k smallest of every query's evaluated WMDs, ordered by (distance, database row): the ka + kb candidates of the
// first rounds (rows idx0, ka + kb per query; distances da, ka per query, then db, kb per query) and the query's list
// [off[j], off[j + 1]) of the rest.  One workgroup per query.
__global__ __launch_bounds__(256) void k_select_lists(const int32_t* __restrict__ idx0, const float* __restrict__ da, int ka,
                                                      const float* __restrict__ db, int kb, int k,
                                                      const int64_t* __restrict__ off, int64_t ja, const int32_t* __restrict__ idx1,
                                                      const float* __restrict__ d1, int32_t* __restrict__ R_idx,
                                                      float* __restrict__ R_dist)
{
    __shared__ float sd[256];
    __shared__ int32_t si[256];
    const int tid = threadIdx.x;
    const int64_t j = ja + blockIdx.x;
    const int64_t a = off[j] - off[ja], cnt = off[j + 1] - off[j];      // idx1 / d1 start at the range's first query
    const int k1 = ka + kb;
    float last_d = -1.f;                 // distances are >= 0, so (-1, -1) precedes every item
    int32_t last_i = -1;
    for (int r = 0; r < k; ++r) {
        float bd = FLT_MAX;
        int32_t bi = INT_MAX;
        for (int64_t e = tid; e < k1 + cnt; e += 256) {
            const float d = e < ka ? da[j * ka + e] : e < k1 ? db[j * kb + e - ka] : d1[a + e - k1];
            const int32_t i = e < k1 ? idx0[j * k1 + e] : idx1[a + e - k1];
            const bool after = d > last_d || (d == last_d && i > last_i);
            if (after && (d < bd || (d == bd && i < bi))) { bd = d; bi = i; }
        }
        sd[tid] = bd;
        si[tid] = bi;
        __syncthreads();
        for (int o = 128; o > 0; o >>= 1) {
            if (tid < o) {
                const float od = sd[tid + o];
                const int32_t oi = si[tid + o];
                if (od < sd[tid] || (od == sd[tid] && oi < si[tid])) { sd[tid] = od; si[tid] = oi; }
            }
            __syncthreads();
        }
        last_d = sd[0];
        last_i = si[0];
        __syncthreads();
        if (tid == 0) { R_idx[j * k + r] = last_i; R_dist[j * k + r] = last_d; }
    }
}

}  // namespace

// -------------------------------------------------------------------------------------------------------------- host
static size_t emd_slab_elems(int64_t h1max, int64_t h2max) { return (size_t)h1max * (size_t)h2max; }

size_t emd_pair_bytes(int64_t h1max, int64_t h2max) { return emd_slab_elems(h1max, h2max) * 12; }   // fp32 costs, fp64 flows

// Words per sink of the map of positive flows, or 0 when the map would take more than 16 KiB of LDS.
static int32_t emd_bitmap_words(int64_t h1max, int64_t h2max)
{
    const int64_t w = (h1max + 31) / 32;
    return w * h2max * 4 <= 16 * 1024 ? (int32_t)w : 0;
}

// Sinks per lane whose state the kernel variant keeps in registers, by the longest query-side histogram: up to 128
// words 2, up to 256 words 4, beyond that 0 (state in LDS).
static int emd_reg_sinks(int64_t h2max) { return h2max <= 128 ? 2 : h2max <= 256 ? 4 : 0; }

// per-word solver state, or the cost tiles when those are larger (the two are never live together)
static size_t emd_lds_bytes(int64_t h1max, int64_t h2max)
{
    // per source 28 bytes (potential, distance, supply, predecessor); per sink 28 (potential, distance, demand, way),
    // 12 in the register variants (demand, way)
    const size_t per_sink = emd_reg_sinks(h2max) ? 12 : 28;
    const size_t state = (size_t)h1max * 28 + (size_t)h2max * per_sink + (size_t)emd_bitmap_words(h1max, h2max) * (size_t)h2max * 4;
    const size_t tiles = (size_t)cost_lds_bytes(emd_slice(emd_reg_sinks(h2max)));
    return state > tiles ? state : tiles;
}

// the settled-node masks hold 32 nodes per lane; the per-word state must fit one workgroup's LDS
bool emd_supported(int64_t h1max, int64_t h2max)
{
    return h1max <= 2048 && h2max <= 2048 && emd_lds_bytes(h1max, h2max) <= 159 * 1024;
}

// Wavefronts that fit the device at once for histograms of this size.

typedef void (*EmdKernel)(const void*, int, int64_t, int32_t, const int64_t*, const int32_t*, const float*, const int64_t*,
                          const int32_t*, const float*, const int32_t*, const int32_t*, int64_t, int32_t*, float*, int64_t,
                          double*, int32_t, int32_t, int32_t, float*, int32_t*, int32_t*, const float*, int32_t, int32_t*);

static EmdKernel emd_kernel(int64_t h2max)
{
    switch (emd_reg_sinks(h2max)) {
    case 2: return k_emd<2>;
    case 4: return k_emd<4>;
    default: return k_emd<0>;
    }
}

int64_t emd_preferred_slots(int num_cu, int64_t h1max, int64_t h2max)
{
    int occ = 0;
    const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, emd_kernel(h2max), 64, emd_lds_bytes(h1max, h2max));
    if (e != hipSuccess || occ < 1) occ = 1;
    return (int64_t)num_cu * occ;
}

// WMD of `count` listed pairs.  `slabs` holds `slots` flow matrices (fp64) followed by `slots` cost matrices (fp32),
// one of each per wavefront of the grid; next_pair is a device counter this call resets.
hipError_t launch_emd(const lcrwmd_emb& E, const lcrwmd_csr& DB, const lcrwmd_csr& Q, const int32_t* pair_db,
                      const int32_t* pair_q, int64_t count, int64_t h1max, int64_t h2max, void* slabs, int64_t slots,
                      int32_t* next_pair, float* out, int32_t* flags, int32_t* fail_count, const float* limit,
                      int32_t limit_j0, int32_t* give_up_count, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    if (slots > count) slots = count;
    const size_t elems = emd_slab_elems(h1max, h2max);
    const size_t lds = emd_lds_bytes(h1max, h2max);
    hipError_t e;
    const EmdKernel kernel = emd_kernel(h2max);
    if (lds > 64 * 1024) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    e = launch_fill_i32(next_pair, 1, 0, s);
    if (e != hipSuccess) return e;
    double* slabs_f = reinterpret_cast<double*>(slabs);
    float* slabs_c = reinterpret_cast<float*>(slabs_f + (size_t)slots * elems);
    const int32_t bmw = emd_bitmap_words(h1max, h2max);
    kernel<<<dim3((unsigned)slots), 64, lds, s>>>(E.data, (int)E.dtype, E.ld, (int32_t)E.m, DB.row_ptr, DB.col_idx, DB.val,
                                                  Q.row_ptr, Q.col_idx, Q.val, pair_db, pair_q, count, next_pair, slabs_c,
                                                  (int64_t)elems, slabs_f, (int32_t)h1max, (int32_t)h2max, bmw, out, flags,
                                                  fail_count, limit, limit_j0, give_up_count);
    return hipGetLastError();
}

hipError_t launch_check_pairs(const int32_t* pair_db, const int32_t* pair_q, int64_t npairs, int64_t n, int64_t q,
                              int32_t* status, hipStream_t s)
{
    if (npairs <= 0) return hipSuccess;
    k_check_pairs<<<dim3((unsigned)((npairs + 255) / 256)), 256, 0, s>>>(pair_db, pair_q, npairs, n, q, status);
    return hipGetLastError();
}

hipError_t launch_centroids(const lcrwmd_emb& E, const lcrwmd_csr& X, float* C, int64_t ldc, hipStream_t s)
{
    if (X.rows <= 0) return hipSuccess;
    k_centroids<<<dim3((unsigned)X.rows), 256, 0, s>>>(E.data, (int)E.dtype, E.ld, (int32_t)E.m, X.row_ptr, X.col_idx,
                                                      X.val, C, ldc);
    return hipGetLastError();
}

hipError_t launch_centroid_dist(const float* C1, int64_t n, const float* C2, int64_t q, int64_t ldc, int32_t m, float* D,
                                int64_t ldd, hipStream_t s)
{
    if (n <= 0 || q <= 0) return hipSuccess;
    const int64_t rows_per_launch = (int64_t)65535 * 64;          // grid.y carries the database rows
    for (int64_t r0 = 0; r0 < n; r0 += rows_per_launch) {
        const int64_t rows = n - r0 < rows_per_launch ? n - r0 : rows_per_launch;
        dim3 grid((unsigned)((q + 63) / 64), (unsigned)((rows + 63) / 64));
        k_centroid_dist<<<grid, 256, 0, s>>>(C1 + r0 * ldc, rows, C2, q, ldc, m, D + r0 * ldd, ldd);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_first_pairs(const int32_t* R0, int64_t q, int stride, int lo, int hi, int32_t j0, float* D, int64_t ldd,
                              int32_t* pair_db, int32_t* pair_q, hipStream_t s)
{
    const int64_t total = q * (hi - lo);
    if (total <= 0) return hipSuccess;
    k_first_pairs<<<dim3((unsigned)((total + 255) / 256)), 256, 0, s>>>(R0, q, stride, lo, hi, j0, D, ldd, pair_db, pair_q);
    return hipGetLastError();
}

hipError_t launch_cutoff(const float* wa, int ka, const float* wb, int kb, int64_t q, int k, float slack, float* cut,
                         hipStream_t s)
{
    if (q <= 0) return hipSuccess;
    k_cutoff<<<dim3((unsigned)((q + 255) / 256)), 256, 0, s>>>(wa, ka, wb, kb, q, k, slack, cut);
    return hipGetLastError();
}

// Survivors per query and their prefix sums off[0..q].  n <= 65535 * 256 rows (the caller checks).
hipError_t launch_count_below(const float* D, int64_t n, int64_t q, int64_t ldd, const float* cut, int32_t* cnt,
                              int64_t* off, hipStream_t s)
{
    if (n <= 0 || q <= 0) return hipSuccess;
    hipError_t e = launch_fill_i32(cnt, q, 0, s);
    if (e != hipSuccess) return e;
    const int64_t row_blocks = (n + kRowsPerBlock - 1) / kRowsPerBlock;
    k_count_below<<<dim3((unsigned)((q + 255) / 256), (unsigned)row_blocks), 256, 0, s>>>(D, n, q, ldd, cut, cnt);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    k_scan_counts<<<1, 1024, 0, s>>>(cnt, q, off);
    return hipGetLastError();
}

// Lists of the survivors of queries [ja, jb), query after query, starting at pair_db[0] / pair_q[0].
hipError_t launch_fill_below(const float* D, int64_t n, int64_t ja, int64_t jb, int64_t ldd, const float* cut,
                             const int64_t* off, int64_t* cursor, int32_t j0, int32_t* pair_db, int32_t* pair_q,
                             hipStream_t s)
{
    if (n <= 0 || jb <= ja) return hipSuccess;
    k_init_cursor<<<dim3((unsigned)((jb - ja + 255) / 256)), 256, 0, s>>>(off, ja, jb, cursor);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t row_blocks = (n + kRowsPerBlock - 1) / kRowsPerBlock;
    k_fill_below<<<dim3((unsigned)((jb - ja + 255) / 256), (unsigned)row_blocks), 256, 0, s>>>(D, n, ja, jb, ldd, cut, cursor,
                                                                                            j0, pair_db, pair_q);
    return hipGetLastError();
}

hipError_t launch_select_lists(const int32_t* idx0, const float* da, int ka, const float* db, int kb, int k, const int64_t* off,
                               int64_t ja, int64_t jb, const int32_t* idx1, const float* d1, int32_t* R_idx, float* R_dist,
                               hipStream_t s)
{
    if (jb <= ja) return hipSuccess;
    k_select_lists<<<dim3((unsigned)(jb - ja)), 256, 0, s>>>(idx0, da, ka, db, kb, k, off, ja, idx1, d1, R_idx, R_dist);
    return hipGetLastError();
}

}  // namespace lcrwmd
