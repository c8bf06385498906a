// C ABI of the LC-RWMD library: argument checks, workspace carving, batching and launch order.
// All arithmetic is in the kernels of the other translation units.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <vector>

#include "lcrwmd_internal.h"

using namespace lcrwmd;

namespace {

lcrwmd_status fail(lcrwmd_ctx* ctx, lcrwmd_status st, const char* fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return st;
}

#define HIP_TRY(expr)                                                                                   \
    do {                                                                                                \
        hipError_t e_ = (expr);                                                                         \
        if (e_ != hipSuccess)                                                                           \
            return fail(ctx, LCRWMD_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_));               \
    } while (0)

#define ST_TRY(expr)                          \
    do {                                      \
        lcrwmd_status s_ = (expr);            \
        if (s_ != LCRWMD_OK) return s_;       \
    } while (0)

// Event bracket around one kernel launch while profiling is on.
struct ProfScope {
    lcrwmd_ctx* ctx;
    hipStream_t s;
    lcrwmd_prof_rec rec;
    bool on;
    ProfScope(lcrwmd_ctx* c, hipStream_t st, int kind, double work, double work2 = 0.0) : ctx(c), s(st), on(false)
    {
        if (!c->profiling) return;
        rec.kind = kind;
        rec.work = work;
        rec.work2 = work2;
        if (hipEventCreate(&rec.start) != hipSuccess) return;
        if (hipEventCreate(&rec.stop) != hipSuccess) { (void)hipEventDestroy(rec.start); return; }
        on = hipEventRecord(rec.start, s) == hipSuccess;
    }
    ~ProfScope()
    {
        if (!on) return;
        (void)hipEventRecord(rec.stop, s);
        ctx->prof.push_back(rec);
    }
};

constexpr int64_t kMaxTokens = (int64_t)1 << 30;   // padded tokens per launch (int32 offsets)
constexpr int64_t kDbBatch = 16384;                // database rows per pass of the swapped direction (option max_db_batch lowers it)

lcrwmd_status check_csr(lcrwmd_ctx* ctx, const lcrwmd_csr* X, const char* name, bool need_val)
{
    if (!X) return fail(ctx, LCRWMD_EINVAL, "%s is NULL", name);
    if (X->rows < 0 || X->cols < 0 || X->nnz < 0) return fail(ctx, LCRWMD_EINVAL, "%s has a negative size", name);
    if (!X->row_ptr) return fail(ctx, LCRWMD_EINVAL, "%s.row_ptr is NULL", name);
    if (X->nnz > 0 && !X->col_idx) return fail(ctx, LCRWMD_EINVAL, "%s.col_idx is NULL", name);
    if (need_val && X->nnz > 0 && !X->val) return fail(ctx, LCRWMD_EINVAL, "%s.val is NULL", name);
    if (X->cols > 0x7fffffffLL) return fail(ctx, LCRWMD_EUNSUPPORTED, "%s.cols exceeds int32", name);
    if (X->rows > 0 && X->nnz < X->rows)
        return fail(ctx, LCRWMD_EEMPTYDOC, "%s stores fewer entries than rows: some histogram is empty", name);
    return LCRWMD_OK;
}

lcrwmd_status check_emb(lcrwmd_ctx* ctx, const lcrwmd_emb* E)
{
    if (!E) return fail(ctx, LCRWMD_EINVAL, "E is NULL");
    if (E->v <= 0 || E->m <= 0) return fail(ctx, LCRWMD_EINVAL, "E must have v > 0 and m > 0");
    if (!E->data) return fail(ctx, LCRWMD_EINVAL, "E.data is NULL");
    if (E->ld < E->m) return fail(ctx, LCRWMD_EINVAL, "E.ld < E.m");
    if (E->dtype != LCRWMD_F32 && E->dtype != LCRWMD_BF16) return fail(ctx, LCRWMD_EINVAL, "unknown E.dtype");
    if (E->v > 0x7fffffffLL || E->m > 65536 || E->ld > 0x7fffffffLL)
        return fail(ctx, LCRWMD_EUNSUPPORTED, "E is too large (v < 2^31, m <= 65536, ld < 2^31)");
    return LCRWMD_OK;
}

lcrwmd_status check_ws(lcrwmd_ctx* ctx, const void* ws, size_t ws_bytes)
{
    if (!ws || ws_bytes == 0) return fail(ctx, LCRWMD_EWORKSPACE, "a workspace is required");
    if (((uintptr_t)ws & 255) != 0) return fail(ctx, LCRWMD_EWORKSPACE, "the workspace must be 256-byte aligned");
    return LCRWMD_OK;
}

bool use_bf16(const lcrwmd_ctx* ctx, const lcrwmd_emb* E) { return E->dtype == LCRWMD_BF16 || ctx->opt.compute == LCRWMD_BF16; }

// Arithmetic of the first phase: 0 fp32, 1 bf16, 2 split bf16 (three products per fp32 product).  The bf16 kernels
// take m <= 300.  Wider embeddings compute in fp32: the split form on E as it is, the bf16 form on an fp32 copy of the
// values as bf16 numbers (products of bf16 values are exact in fp32, so the results are those the bf16 form defines).
int prec_mode(const lcrwmd_ctx* ctx, const lcrwmd_emb* E)
{
    if (E->m > 300) return 0;
    if (use_bf16(ctx, E)) return 1;
    if (ctx->opt.compute == LCRWMD_BF16X3) return 2;
    return 0;
}

// bf16 was asked for (storage or compute option) but the embeddings are too wide for the bf16 kernels
bool wants_widened_copy(const lcrwmd_ctx* ctx, const lcrwmd_emb* E) { return E->m > 300 && use_bf16(ctx, E); }

lcrwmd_status validate_on_device(lcrwmd_ctx* ctx, const lcrwmd_csr* X, const char* name, int32_t* dev_status,
                                 hipStream_t s)
{
    HIP_TRY(launch_fill_i32(dev_status, 1, 0, s));
    HIP_TRY(launch_validate_csr(*X, dev_status, s));
    int32_t h = 0;
    HIP_TRY(hipMemcpyAsync(&h, dev_status, sizeof(h), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (h == LCRWMD_EEMPTYDOC) return fail(ctx, LCRWMD_EEMPTYDOC, "%s contains an empty histogram", name);
    if (h != 0) return fail(ctx, LCRWMD_EBADCSR, "%s is not a valid CSR matrix (row_ptr, column order/range or weights)", name);
    return LCRWMD_OK;
}

// Embedding operand prepared for the first phase: squared norms, and for bf16 the packed copy.
struct EmbPrep {
    const void* data;
    int64_t ld;
    int64_t rows;  // rows of `data`
    int32_t m;     // embedding dimension the first-phase kernels are told (300 for the padded fp32 copy)
    float* normE;
    bool bf16;     // mode 1
    int mode;      // see prec_mode
    // the same values for the pass that redoes close word pairs from coordinate differences (launch_redo_close)
    const void* xdata;
    int64_t xld;
    int32_t xm;
    bool xbf16;
};

// fp32 E that the tile kernel cannot read in place (a pitch or base that is not 16-byte aligned, or 200 < m < 300):
// a zero-padded copy with the shape that kernel takes (300 columns, 304 floats per row) is cheaper than the general
// kernels, which reach 50-58 % of peak: measured crossover near m = 190.
constexpr int32_t kPadM = 300, kPadPitch = 304, kPadFromM = 208;

bool wants_padded_copy(const lcrwmd_emb* E)
{
    if (E->dtype != LCRWMD_F32 || E->m > kPadM || E->m < kPadFromM) return false;
    Phase1Args a;
    a.E = E->data;
    a.ld = E->ld;
    a.erows = E->v;
    a.m = (int32_t)E->m;
    return !tiles_f32_supported(a) && tiles_rows_addressable(E->v, (int64_t)kPadPitch * 4);
}

// padded: room for the zero-padded fp32 copy (wants_padded_copy; the public size query, which does not know E's
// address, counts it for every width that may need it)
// widened: room for the fp32 copy of bf16-valued embeddings wider than the bf16 kernels take
size_t emb_prep_bytes(int64_t v, int32_t m, int mode, bool padded, bool widened = false)
{
    return (size_t)v * 4 + 256 +
           (mode == 1 ? pack_bf16_bytes(v, m) + 256
            : mode == 2 ? pack_x3_bytes(v) + 256
            : padded ? (size_t)v * kPadPitch * 4 + 256
            : widened ? (size_t)v * (size_t)m * 4 + 256 : 0);
}

lcrwmd_status prepare_emb(lcrwmd_ctx* ctx, const lcrwmd_emb* E, Bump& b, EmbPrep& ep, hipStream_t s)
{
    ep.mode = prec_mode(ctx, E);
    ep.bf16 = ep.mode == 1;
    ep.m = (int32_t)E->m;
    ep.rows = E->v;
    if (ep.mode != 0 && !tiles_rows_addressable(E->v, ep.mode == 1 ? bf16_pitch((int32_t)E->m) * 2 : x3_pitch() * 2))
        return fail(ctx, LCRWMD_EUNSUPPORTED, "E has too many rows for the bf16 kernels' packed copy (64 GiB limit)");
    ep.normE = b.take_n<float>((size_t)E->v);
    if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for the word norms");
    if (ep.mode == 2) {
        void* packed = b.take(pack_x3_bytes(E->v));
        if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for the split copy of E");
        HIP_TRY(launch_pack_x3((const float*)E->data, E->v, (int32_t)E->m, E->ld, packed, ep.normE, s));
        ep.data = packed;
        ep.ld = x3_pitch();
        ep.xdata = E->data;             // hi + lo stands for the fp32 value
        ep.xld = E->ld;
        ep.xm = (int32_t)E->m;
        ep.xbf16 = false;
        return LCRWMD_OK;
    }
    if (ep.bf16) {
        void* packed = b.take(pack_bf16_bytes(E->v, (int32_t)E->m));
        if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for the bf16 copy of E");
        HIP_TRY(launch_pack_bf16(E->data, E->dtype, E->v, (int32_t)E->m, E->ld, packed, ep.normE, s));
        ep.data = packed;
        ep.ld = bf16_pitch((int32_t)E->m);
    } else if (wants_widened_copy(ctx, E)) {
        float* wide = b.take_n<float>((size_t)E->v * (size_t)E->m);
        if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for the fp32 copy of the wide embeddings");
        HIP_TRY(launch_widen_bf16(E->data, E->dtype, E->v, (int32_t)E->m, E->ld, wide, s));
        HIP_TRY(launch_row_norms_f32(wide, E->v, (int32_t)E->m, E->m, ep.normE, s));
        ep.data = wide;
        ep.ld = E->m;
    } else {
        if (wants_padded_copy(E)) {
            Bump saved = b;
            float* packed = b.take_n<float>((size_t)E->v * kPadPitch);
            if (b.ok) {
                HIP_TRY(launch_pack_f32((const float*)E->data, E->v, (int32_t)E->m, E->ld, kPadPitch, packed, ep.normE, s));
                ep.data = packed;
                ep.ld = kPadPitch;
                ep.m = kPadM;
                ep.xdata = packed;
                ep.xld = kPadPitch;
                ep.xm = (int32_t)E->m;
                ep.xbf16 = false;
                return LCRWMD_OK;
            }
            b = saved;                  // no room for the copy: the general kernels read E in place
        }
        HIP_TRY(launch_row_norms_f32((const float*)E->data, E->v, (int32_t)E->m, E->ld, ep.normE, s));
        ep.data = E->data;
        ep.ld = E->ld;
    }
    ep.xdata = ep.data;                 // fp32 rows, or the packed bf16 rows (values first)
    ep.xld = ep.ld;
    ep.xm = (int32_t)E->m;
    ep.xbf16 = ep.bf16;
    return LCRWMD_OK;
}

// One first-phase pass over histograms [r0, r0 + nseg) of a CSR whose row_ptr is `rp` (device).
// Room for the contraction kernel's map of close pairs, when the workspace has it (nullptr otherwise: the pass that
// redoes close pairs then reads all of Z to find them).
uint64_t* take_close_bits(Bump& b, int64_t nseg, int64_t nvoc)
{
    Bump saved = b;
    void* p = b.take(close_bits_bytes(nseg, nvoc));
    if (!b.ok) { b = saved; return nullptr; }
    return (uint64_t*)p;
}

lcrwmd_status run_phase1(lcrwmd_ctx* ctx, const EmbPrep& ep, int32_t m, const int32_t* voc_rows, int64_t nvoc,
                         int z_by_position, const int32_t* zero_map, const int64_t* rp_batch,
                         const int32_t* col_idx, int64_t tokens, const TokenPlan& tp, float* Z, int64_t ldz,
                         hipStream_t s, bool swapped = false, uint64_t* close_bits = nullptr)
{
    HIP_TRY(launch_token_plan(tp, rp_batch, col_idx, ep.normE, s));
    Phase1Args a;
    a.E = ep.data;
    a.ld = ep.ld;
    a.erows = ep.rows;
    a.m = ep.m;                 // what the kernel multiplies; the flop count below uses the caller's m
    a.normE = ep.normE;
    a.voc_rows = voc_rows;
    a.nvoc = nvoc;
    a.z_by_position = z_by_position;
    a.Z = Z;
    a.ldz = ldz;
    a.num_cu = ctx->num_cu;
    // only the tile kernels write the map of close pairs (all bf16 and split-bf16 launches; fp32 where its shape allows)
    const bool mapped = close_bits && (ep.mode != 0 || tiles_f32_supported(a));
    a.close_bits = mapped ? close_bits : nullptr;
    {
        ProfScope ps(ctx, s, 1, 2.0 * (double)nvoc * (double)tokens * (double)m, swapped ? 1.0 : 0.0);
        if (ep.mode == 2) HIP_TRY(launch_phase1_tiles_x3(a, tp, s));
        else if (ep.bf16) HIP_TRY(launch_phase1_bf16(a, tp, s));
        else HIP_TRY(launch_phase1_f32(a, tp, s));
    }
    // a word that occurs in the histogram is at distance exactly 0 from it; the norm expansion
    // only gets there up to cancellation error.  (A vocabulary that lists words more than once - the stacked
    // histograms of the quadratic method - has no word -> row map: the pass below finds those entries itself.)
    if (!voc_rows || zero_map)
        HIP_TRY(launch_zero_matches(rp_batch, col_idx, tp.nseg, zero_map, Z, ldz, s, mapped ? close_bits : nullptr,
                                    close_bits_pitch(ep.mode, nvoc), close_bits_slice(ep.mode)));
    // ... and loses relative accuracy where two different words lie close together: those entries are redone
    if (mapped)
        HIP_TRY(launch_redo_close_bits(ep.xdata, ep.xbf16, ep.xld, ep.xm, voc_rows, nvoc, rp_batch, col_idx, tp.nseg, Z, ldz, close_bits,
                                       close_bits_pitch(ep.mode, nvoc), close_bits_slice(ep.mode), s));
    else
        HIP_TRY(launch_redo_close(ep.xdata, ep.xbf16, ep.xld, ep.xm, ep.normE, voc_rows, nvoc, rp_batch, col_idx, tp.nseg, Z, ldz, s));
    return LCRWMD_OK;
}

// Second-phase launch with its algorithmic traffic: CSR arrays, `zrows` rows of Z, and the output once
// (twice when it is read back for a maximum).
// zrows: rows of Z; z_counted: whether this launch is the one that counts Z's bytes (a Z shared by the launches of
// several blocks of rows is algorithmically read once)
lcrwmd_status run_spmm(lcrwmd_ctx* ctx, const int64_t* rp, const int32_t* ci, const float* xv, int64_t rows,
                       int64_t nnz, int64_t zrows, const float* Z, int64_t ldz, int64_t ncols, float* D, int64_t ldd,
                       int combine, hipStream_t s, bool z_counted = true)
{
    const double bytes = 8.0 * (double)nnz + 8.0 * (double)(rows + 1) + (z_counted ? 4.0 * (double)ncols * (double)zrows : 0.0) +
                         (combine ? 8.0 : 4.0) * (double)ncols * (double)rows;
    ProfScope ps(ctx, s, 2, bytes, 4.0 * (double)nnz * (double)ncols);
    HIP_TRY(launch_spmm(rp, ci, xv, rows, Z, ldz, zrows, ncols, D, ldd, combine, s));
    return LCRWMD_OK;
}

int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }


// Vocabulary tile count the token plan sizes its chunks for (it aims at a few thousand (tile, chunk) pairs).  The
// bf16 kernel balances its load in units of chunks, so it gets eight times as many, shorter chunks.
int64_t plan_tiles(int64_t nvt, bool bf16) { return bf16 ? (nvt + 7) / 8 : nvt; }

// Fixed part of the workspace of lcrwmd_rwmd (everything but the per-batch region).
size_t rwmd_fixed_bytes(int64_t v, int32_t m, int64_t nnz_q, int64_t nnz_db, int mode, bool padded, bool widened = false)
{
    size_t b = emb_prep_bytes(v, m, mode, padded, widened);
    b += 4 * ((size_t)v * 4 + 256);           // flags, word list of the database, word -> position maps of both sets
    b += (size_t)(v < nnz_q ? v : nnz_q) * 4 + 256;   // word list of the queries
    b += (size_t)nnz_q * 4 + 256;             // query columns renumbered to positions
    b += (size_t)nnz_db * 4 + 256;            // database columns renumbered to positions
    b += 1024;                                // counters
    return b;
}

size_t rev_batch_bytes(int64_t vq, int64_t nb, int64_t tokens)
{
    return token_plan_bytes(nb, tokens) + (size_t)vq * (size_t)round_up(nb, 4) * 4 + 256;
}

struct HostPtr {   // host copy of a row_ptr array, borrowed or owned
    const int64_t* p = nullptr;
    std::vector<int64_t> own;
};

lcrwmd_status host_row_ptr(lcrwmd_ctx* ctx, const lcrwmd_csr* X, HostPtr& out, hipStream_t s)
{
    if (X->row_ptr_host) { out.p = X->row_ptr_host; return LCRWMD_OK; }
    try {
        out.own.resize((size_t)X->rows + 1);
    } catch (const std::bad_alloc&) {
        return fail(ctx, LCRWMD_EINVAL, "out of host memory for a row_ptr copy");
    }
    HIP_TRY(hipMemcpyAsync(out.own.data(), X->row_ptr, sizeof(int64_t) * ((size_t)X->rows + 1),
                           hipMemcpyDeviceToHost, s));
    out.p = out.own.data();
    return LCRWMD_OK;
}

// Exact padded token count of histograms [a, b): every histogram rounded up to a multiple of `group` tokens.
int64_t padded_tokens(const int64_t* rp, int64_t a, int64_t b, int group)
{
    int64_t t = 0;
    for (int64_t r = a; r < b; ++r) t += (rp[r + 1] - rp[r] + (group - 1)) & ~(int64_t)(group - 1);
    return t;
}

// Group size of the token plan: the kernel of the split-bf16 arithmetic takes segments padded to 4 tokens, all others
// to 8.
int plan_group(const EmbPrep& ep) { return ep.mode == 2 ? phase1_group_x3() : kGroup; }

// Chunk length limit of the token plan: short where the kernel that walks runs of chunks will run (bf16 and split
// bf16 always; fp32 where its operand shape allows), long for the other fp32 kernels.
int plan_chunk_tiles(const EmbPrep& ep)
{
    if (ep.mode != 0) return kShortChunkTiles;
    Phase1Args a;
    a.E = ep.data;
    a.ld = ep.ld;
    a.erows = ep.rows;
    a.m = ep.m;
    return tiles_f32_supported(a) ? kShortChunkTiles : kLongChunkTiles;
}

int64_t max_tokens_per_batch(const int64_t* rp, int64_t rows, int64_t batch)
{
    int64_t mx = 0;
    for (int64_t a = 0; a < rows; a += batch) {
        int64_t b = a + batch < rows ? a + batch : rows;
        if (rp[b] - rp[a] > mx) mx = rp[b] - rp[a];
    }
    return mx;
}

// What becomes of the bound of a block of database rows once both directions are in it (the top-k of
// lcrwmd_rwmd_reduce, its column sums): tile is (i1 - i0) x q with pitch ldt, row r of it is database row i0 + r.
struct TileSink {
    virtual lcrwmd_status consume(int64_t i0, int64_t i1, const float* tile, int64_t ldt, hipStream_t s) = 0;
    virtual ~TileSink() {}
};

// Which of the two forms is expected to be faster.  Rates measured on one MI355X (kernel times of the five benchmark
// workloads): first-phase contraction in algorithmic flop/s per arithmetic; table passes in table bytes/s, lane
// iterations/s of the per-query loop of the swapped table pass and LDS look-ups/s of the forward table pass.
bool table_form_is_faster(int mode, int32_t m, int64_t ve, int64_t vq, int64_t n, int64_t nnz_db, int64_t q, int64_t nnz_q)
{
    const double rate_p1 = mode == 1 ? 1.2e15 : mode == 2 ? 4.3e14 : 1.37e14;
    const double rate_tab = mode == 1 ? 1.0e15 : mode == 2 ? 2.8e14 : 1.17e14;
    int32_t wcols, nstrip;
    table_strips(vq, &wcols, &nstrip);
    const double per_entry = 2.0 * m * ((double)ve * (double)nnz_q + (double)vq * (double)nnz_db) / rate_p1;
    const double table = 2.0 * m * (double)ve * (double)vq / rate_tab + 4.0 * (double)nnz_db * (double)vq / 1.2e13 +
                         (double)n * (double)q * (double)nstrip / 2.8e11 + (double)ve * (double)nnz_q / 1.3e12 +
                         4.0 * (double)ve * (double)vq / 4.0e12;
    return table < per_entry;
}

// The whole bound for the query rows [jq0, jq1) of Q against the database: into D (n x (jq1 - jq0), ldd) when sink is
// null, else block of database rows by block into a tile of the workspace that is handed to the sink and never
// written anywhere else.  rq / rdb are host copies of the two row_ptr arrays.
//
// Order of work (Sec. IV, many-to-many form, both directions): vocabulary reduction of both sets; forward first phase
// for all queries of the range (Z: one row per database word, one column per query; per-entry form: contraction +
// minimum in batches of queries; table form: one word-pair table, minima looked up); then per block of database rows
//   forward second phase   tile  = X1[block] * Z
//   swapped first phase    Z'    = minima of the query words against the block's histograms (per-entry form)
//   swapped second phase   tile  = max(tile, (X2 * Z')^T)        (table form: both steps from the table)
// so a block's tile is produced, completed and consumed while it is cache resident.
// Returns LCRWMD_EWORKSPACE with *shrink = true when the range's Z does not fit and a smaller range could.
// db_row0: first database row of the bound (the all-pairs job within one set skips the rows before its batch).
lcrwmd_status rwmd_core(lcrwmd_ctx* ctx, const lcrwmd_csr* Q, const int64_t* rq, int64_t jq0, int64_t jq1,
                        const lcrwmd_csr* DB, const int64_t* rdb, const lcrwmd_emb* E, float* D, int64_t ldd,
                        TileSink* sink, void* ws, size_t ws_bytes, hipStream_t s, bool* shrink, int64_t db_row0 = 0)
{
    const int64_t v = E->v, n = DB->rows, q = jq1 - jq0;
    const int64_t qoff = rq[jq0], nnz_q = rq[jq1] - rq[jq0];
    const int32_t m = (int32_t)E->m;
    if (shrink) *shrink = false;
    Bump b(ws, ws_bytes);

    int32_t* counters = b.take_n<int32_t>(64);
    EmbPrep ep;
    ST_TRY(prepare_emb(ctx, E, b, ep, s));

    // Vocabulary reduction (Sec. IV): the forward pass needs only the words of the database, the
    // swapped pass only the words of the queries.
    int32_t* flags = b.take_n<int32_t>((size_t)v);
    int32_t* list_db = b.take_n<int32_t>((size_t)v);
    int32_t* map_db = b.take_n<int32_t>((size_t)v);
    int32_t* dbcol_pos = b.take_n<int32_t>((size_t)DB->nnz);
    int32_t* map_q = b.take_n<int32_t>((size_t)v);
    int32_t* list_q = b.take_n<int32_t>((size_t)(v < nnz_q ? v : nnz_q));
    int32_t* qcol_pos = b.take_n<int32_t>((size_t)nnz_q);
    if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for the vocabulary maps");

    // the database's words: those of the rows the bound covers (all of them unless db_row0 says otherwise)
    const int64_t e0 = rdb[db_row0], nnz_used = DB->nnz - e0;
    HIP_TRY(launch_fill_i32(flags, v, 0, s));
    HIP_TRY(launch_mark_words(DB->col_idx + e0, nnz_used, flags, s));
    HIP_TRY(launch_compact_words(flags, v, list_db, map_db, counters + 0, s));
    HIP_TRY(launch_remap_cols(DB->col_idx + e0, nnz_used, map_db, dbcol_pos + e0, s));
    HIP_TRY(launch_fill_i32(flags, v, 0, s));
    HIP_TRY(launch_mark_words(Q->col_idx + qoff, nnz_q, flags, s));
    HIP_TRY(launch_compact_words(flags, v, list_q, map_q, counters + 1, s));
    HIP_TRY(launch_remap_cols(Q->col_idx + qoff, nnz_q, map_q, qcol_pos, s));

    int32_t hc[2] = {0, 0};
    HIP_TRY(hipMemcpyAsync(hc, counters, sizeof(hc), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));          // the vocabulary sizes decide grids and batch sizes
    const int64_t ve = hc[0], vq = hc[1];

    // Z of the whole range: one row per database word
    const int64_t ldz = round_up(q, 4);
    float* Z = b.take_n<float>((size_t)ve * ldz);
    const size_t region_off = (b.used + 255) & ~(size_t)255;
    if (!b.ok || region_off >= b.size) {
        if (shrink) *shrink = q > 1;
        return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for the first-phase minima of %lld queries", (long long)q);
    }
    const size_t region = b.size - region_off;
    const int grp = plan_group(ep), chunk_tiles = plan_chunk_tiles(ep);
    int64_t nb_max = n < kDbBatch ? n : kDbBatch;
    if (ctx->opt.max_db_batch > 0 && nb_max > ctx->opt.max_db_batch) nb_max = ctx->opt.max_db_batch;
    const size_t tile_row = sink ? (size_t)ldz * 4 : 0;          // a block's tile lives in the workspace when there is a sink

    // ---- table form: one word-pair table for the range, both directions read it ----
    bool table = false;
    if (ctx->opt.dedup && ve > 0 && vq > 0 && q <= table_max_queries() &&
        (ctx->opt.dedup == 1 || table_form_is_faster(ep.mode, m, ve, vq, n - db_row0, nnz_used, q, nnz_q))) {
        Phase1Args a;
        a.E = ep.data;
        a.ld = ep.ld;
        a.erows = ep.rows;
        a.m = ep.m;
        a.normE = ep.normE;
        a.z_by_position = 1;
        // columns of the table: the query words dealt out over the column strips (vc places, a few of them unused)
        int32_t ws_cols, nstrip;
        table_strips(vq, &ws_cols, &nstrip);
        const int64_t vc = (int64_t)ws_cols * nstrip;
        const int64_t ldw = vc;                                      // ws_cols is a multiple of 32: rows start on 128-byte lines
        const int64_t tok_count = round_up(ve, kTileTokens) + kTileTokens;
        Bump bb(b.base + region_off, region);
        float* W = bb.take_n<float>((size_t)ve * ldw);
        int32_t* tok_ids = bb.take_n<int32_t>((size_t)tok_count);
        float* tok_hn = bb.take_n<float>((size_t)tok_count);
        const size_t nsq = (size_t)nstrip * (size_t)q + 1;
        int32_t* bcnt = bb.take_n<int32_t>(nsq);
        int32_t* boffs = bb.take_n<int32_t>(nsq);
        int32_t* bcur = bb.take_n<int32_t>(nsq);
        int32_t* bpos = bb.take_n<int32_t>((size_t)nnz_q);
        float* bval = bb.take_n<float>((size_t)nnz_q);
        int32_t* col_word = bb.take_n<int32_t>((size_t)vc);
        int32_t* qcol = bb.take_n<int32_t>((size_t)nnz_q);
        // per block of database rows: partial sums between the strips, and the tile when a sink takes it
        // (without a sink all rows go in one block: a strip of the table is then streamed once per call, not once
        // per block)
        int64_t nb = sink ? nb_max : n;
        const size_t per_row = (nstrip > 1 ? (size_t)ldz * 4 : 0) + tile_row;
        if (per_row > 0 && bb.ok) {
            const size_t room = bb.size - ((bb.used + 255) & ~(size_t)255);
            const int64_t fit = (int64_t)((room > 1024 ? room - 1024 : 0) / per_row);
            if (fit < nb) nb = fit;
        }
        a.voc_rows = col_word;
        a.nvoc = vc;
        a.Z = W;
        a.ldz = ldw;
        if (bb.ok && nb >= 1 && distance_table_supported(a, ep.mode)) {
            float* D2 = nstrip > 1 ? bb.take_n<float>((size_t)nb * ldz) : nullptr;
            float* tile = sink ? bb.take_n<float>((size_t)nb * ldz) : nullptr;
            table = true;
            ctx->forms_ran |= 2;
            HIP_TRY(launch_table_spread(list_q, vq, qcol_pos, nnz_q, col_word, qcol, s));
            HIP_TRY(launch_table_tokens(list_db, ve, ep.normE, tok_ids, tok_hn, tok_count, s));
            {
                ProfScope ps(ctx, s, 1, 2.0 * (double)ve * (double)vq * (double)m);
                HIP_TRY(launch_distance_table(a, ep.mode, tok_ids, tok_hn, ve, s));
            }
            HIP_TRY(launch_table_zero_same(col_word, vc, map_db, W, ldw, s));
            HIP_TRY(launch_table_redo_close(ep.xdata, ep.xbf16, ep.xld, ep.xm, ep.normE, list_db, ve, col_word, vc, W, ldw, s));
            HIP_TRY(launch_table_buckets(Q->row_ptr + jq0, qcol - qoff, Q->val, q, vc, bcnt, boffs, bcur, bpos, bval, s));
            {   // forward: every table row once, Z once
                ProfScope ps(ctx, s, 3, 4.0 * (double)ve * (double)vq + 4.0 * (double)ve * (double)q + 8.0 * (double)nnz_q);
                HIP_TRY(launch_table_fwd(W, ldw, ve, vc, boffs, bpos, q, Z, ldz, s));
            }
            for (int64_t i0 = db_row0; i0 < n; i0 += nb) {
                const int64_t i1 = i0 + nb < n ? i0 + nb : n;
                const int64_t nnz_b = rdb[i1] - rdb[i0];
                float* Db = sink ? tile : D + i0 * ldd;
                const int64_t ldb = sink ? ldz : ldd;
                ST_TRY(run_spmm(ctx, DB->row_ptr + i0, dbcol_pos, DB->val, i1 - i0, nnz_b, ve, Z, ldz, q, Db, ldb, 0, s, i0 == db_row0));
                {   // swapped: one table row per stored database entry, the block read and written once
                    ProfScope ps(ctx, s, 4, 4.0 * (double)nnz_b * (double)vq + 8.0 * (double)(i1 - i0) * (double)q + 4.0 * (double)nnz_b);
                    HIP_TRY(launch_table_rev(W, ldw, vc, DB->row_ptr + i0, dbcol_pos, i1 - i0, boffs, bpos, bval, q, D2, ldz, Db, ldb, s));
                }
                if (sink) ST_TRY(sink->consume(i0, i1, Db, ldb, s));
            }
            return LCRWMD_OK;
        }
        // the table does not fit the workspace (or the embedding shape has no table kernel): per-entry form below
    }
    (void)table;
    ctx->forms_ran |= 1;

    // ---- forward first phase: Z[p][j] = min over the words of query j of the distance to database word p ----
    {
        int64_t qb = q;
        if (ctx->opt.max_query_batch > 0 && qb > ctx->opt.max_query_batch) qb = ctx->opt.max_query_batch;
        for (;;) {
            int64_t tok = max_tokens_per_batch(rq + jq0, q, qb);
            if (tok + 7 * qb < kMaxTokens && token_plan_bytes(qb, tok) <= region) break;
            if (qb == 1) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for one query (forward pass)");
            qb = (qb + 1) / 2;
        }
        const int64_t nvt_f = (ve + kTileVocab - 1) / kTileVocab;
        for (int64_t j0 = jq0; j0 < jq1; j0 += qb) {
            const int64_t j1 = j0 + qb < jq1 ? j0 + qb : jq1;
            Bump bb(b.base + region_off, region);
            TokenPlan tp;
            carve_token_plan(bb, tp, j1 - j0, rq[j1] - rq[j0], plan_tiles(nvt_f, ep.bf16), padded_tokens(rq, j0, j1, grp), grp,
                             chunk_tiles);
            if (!bb.ok) return fail(ctx, LCRWMD_EWORKSPACE, "internal: forward batch does not fit");
            uint64_t* bits = take_close_bits(bb, j1 - j0, ve);
            ST_TRY(run_phase1(ctx, ep, m, list_db, ve, /*z_by_position=*/1, /*zero_map=*/map_db, Q->row_ptr + j0,
                              Q->col_idx, rq[j1] - rq[j0], tp, Z + (j0 - jq0), ldz, s, false, bits));
        }
    }

    // ---- per block of database rows: forward second phase, swapped first and second phase, D = max(D1, D2^T) ----
    int64_t nb = nb_max;
    for (;;) {
        int64_t tok = max_tokens_per_batch(rdb + db_row0, n - db_row0, nb);
        if (tok + 7 * nb < kMaxTokens && rev_batch_bytes(vq, nb, tok) + (size_t)nb * tile_row + 256 <= region) break;
        if (nb == 1) {
            if (shrink) *shrink = q > 1;
            return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for one database row (swapped pass)");
        }
        nb = (nb + 1) / 2;
    }
    const int64_t nvt_r = (vq + kTileVocab - 1) / kTileVocab;
    for (int64_t i0 = db_row0; i0 < n; i0 += nb) {
        const int64_t i1 = i0 + nb < n ? i0 + nb : n;
        const int64_t nnz_b = rdb[i1] - rdb[i0];
        Bump bb(b.base + region_off, region);
        TokenPlan tp;
        carve_token_plan(bb, tp, i1 - i0, nnz_b, plan_tiles(nvt_r, ep.bf16), padded_tokens(rdb, i0, i1, grp), grp, chunk_tiles);
        const int64_t ldzr = round_up(i1 - i0, 4);
        float* Zr = bb.take_n<float>((size_t)vq * ldzr);
        float* tile = sink ? bb.take_n<float>((size_t)(i1 - i0) * ldz) : nullptr;
        if (!bb.ok) return fail(ctx, LCRWMD_EWORKSPACE, "internal: block of database rows does not fit");
        uint64_t* bits = take_close_bits(bb, i1 - i0, vq);
        float* Db = sink ? tile : D + i0 * ldd;
        const int64_t ldb = sink ? ldz : ldd;
        ST_TRY(run_spmm(ctx, DB->row_ptr + i0, dbcol_pos, DB->val, i1 - i0, nnz_b, ve, Z, ldz, q, Db, ldb, 0, s, i0 == db_row0));
        ST_TRY(run_phase1(ctx, ep, m, list_q, vq, /*z_by_position=*/1, /*zero_map=*/map_q, DB->row_ptr + i0,
                          DB->col_idx, nnz_b, tp, Zr, ldzr, s, /*swapped=*/true, bits));
        // the queries' row_ptr holds offsets into the caller's arrays; shift the renumbered columns to match
        ST_TRY(run_spmm(ctx, Q->row_ptr + jq0, qcol_pos - qoff, Q->val, q, nnz_q, vq, Zr, ldzr, i1 - i0, Db, ldb, 2, s));
        if (sink) ST_TRY(sink->consume(i0, i1, Db, ldb, s));
    }
    return LCRWMD_OK;
}

// rwmd_core over all queries: the whole set at once when its first-phase minima fit the workspace (and the table
// kernels' limit on queries per pass, when the table form may run), otherwise in ranges of queries.
lcrwmd_status rwmd_ranges(lcrwmd_ctx* ctx, const lcrwmd_csr* Q, const int64_t* rq, const lcrwmd_csr* DB, const int64_t* rdb,
                          const lcrwmd_emb* E, float* D, int64_t ldd, int64_t qr, void* ws, size_t ws_bytes, hipStream_t s)
{
    const int64_t q = Q->rows;
    if (qr > q) qr = q;
    if (ctx->opt.dedup == 1 && qr > table_max_queries()) qr = table_max_queries();
    for (int64_t j0 = 0; j0 < q;) {
        const int64_t j1 = j0 + qr < q ? j0 + qr : q;
        bool shrink = false;
        lcrwmd_status st = rwmd_core(ctx, Q, rq, j0, j1, DB, rdb, E, D + j0, ldd, nullptr, ws, ws_bytes, s, &shrink);
        if (st == LCRWMD_EWORKSPACE && shrink && qr > 1) { qr = (qr + 1) / 2; continue; }    // nothing of this range was written
        if (st != LCRWMD_OK) return st;
        j0 = j1;
    }
    return LCRWMD_OK;
}

// Host row pointers of both sets (one synchronisation when a copy has to be fetched) and optional validation.
lcrwmd_status fetch_rows_and_validate(lcrwmd_ctx* ctx, const lcrwmd_csr* Q, const lcrwmd_csr* DB, HostPtr& rq,
                                      HostPtr& rdb, void* ws, size_t ws_bytes, hipStream_t s)
{
    if (ctx->opt.validate) {
        Bump b(ws, ws_bytes);
        int32_t* st = b.take_n<int32_t>(64);
        if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small");
        ST_TRY(validate_on_device(ctx, Q, "queries", st, s));
        ST_TRY(validate_on_device(ctx, DB, "database", st, s));
    }
    ST_TRY(host_row_ptr(ctx, Q, rq, s));
    ST_TRY(host_row_ptr(ctx, DB, rdb, s));
    if (!Q->row_ptr_host || !DB->row_ptr_host) HIP_TRY(hipStreamSynchronize(s));
    if (rq.p[0] != 0 || rq.p[Q->rows] != Q->nnz || rdb.p[0] != 0 || rdb.p[DB->rows] != DB->nnz)
        return fail(ctx, LCRWMD_EBADCSR, "row_ptr does not span [0, nnz]");
    for (int64_t r = 0; r < Q->rows; ++r)
        if (rq.p[r + 1] <= rq.p[r]) return fail(ctx, LCRWMD_EEMPTYDOC, "queries row %lld is empty or row_ptr decreases", (long long)r);
    for (int64_t r = 0; r < DB->rows; ++r)
        if (rdb.p[r + 1] <= rdb.p[r]) return fail(ctx, LCRWMD_EEMPTYDOC, "database row %lld is empty or row_ptr decreases", (long long)r);
    return LCRWMD_OK;
}

lcrwmd_status check_rwmd_args(lcrwmd_ctx* ctx, const lcrwmd_csr* Q, const lcrwmd_csr* DB, const lcrwmd_emb* E)
{
    ST_TRY(check_emb(ctx, E));
    ST_TRY(check_csr(ctx, Q, "queries", true));
    ST_TRY(check_csr(ctx, DB, "database", true));
    if (Q->cols != E->v || DB->cols != E->v) return fail(ctx, LCRWMD_EINVAL, "histogram columns must equal E.v");
    return LCRWMD_OK;
}

}  // namespace

extern "C" {

lcrwmd_status lcrwmd_create(lcrwmd_ctx** out, int device)
{
    if (!out) return LCRWMD_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return LCRWMD_EHIP;
    lcrwmd_ctx* c = new (std::nothrow) lcrwmd_ctx();
    if (!c) return LCRWMD_EINVAL;
    c->err[0] = 0;
    c->profiling = false;
    c->opt = lcrwmd_options{0, LCRWMD_F32, 0, 0, 0};
    c->device = device;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) { delete c; return LCRWMD_EHIP; }
    c->num_cu = prop.multiProcessorCount;
    c->device_bytes = prop.totalGlobalMem;
    // this device's address of the scratch array behind lcrwmd_topk_noalloc (looked up with the device current)
    if (hipSetDevice(device) != hipSuccess || topk_static_init(device) != hipSuccess) { delete c; return LCRWMD_EHIP; }
    c->opt.validate = 0;
    c->opt.compute = LCRWMD_F32;
    *out = c;
    return LCRWMD_OK;
}

void lcrwmd_destroy(lcrwmd_ctx* ctx)
{
    if (!ctx) return;
    for (auto& r : ctx->prof) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    delete ctx;
}

lcrwmd_status lcrwmd_profile_begin(lcrwmd_ctx* ctx)
{
    if (!ctx) return LCRWMD_EINVAL;
    for (auto& r : ctx->prof) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    ctx->prof.clear();
    ctx->prof_abandoned = 0.0;
    ctx->profiling = true;
    return LCRWMD_OK;
}

lcrwmd_status lcrwmd_profile_end(lcrwmd_ctx* ctx, lcrwmd_profile* out)
{
    if (!ctx) return LCRWMD_EINVAL;
    if (!out) return fail(ctx, LCRWMD_EINVAL, "out is NULL");
    ctx->profiling = false;
    memset(out, 0, sizeof(*out));
    HIP_TRY(hipSetDevice(ctx->device));
    HIP_TRY(hipDeviceSynchronize());
    for (auto& r : ctx->prof) {
        float ms = 0.f;
        hipError_t e = hipEventElapsedTime(&ms, r.start, r.stop);
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
        if (e != hipSuccess) continue;
        if (r.kind == 1) {
            out->phase1_ms += ms;
            out->phase1_launches += 1;
            out->phase1_flops += r.work;
            if (r.work2 > 0.0) { out->phase1_swapped_ms += ms; out->phase1_swapped_flops += r.work; }
        }
        else if (r.kind == 3) { out->table_fwd_ms += ms; out->table_fwd_launches += 1; out->table_fwd_bytes += r.work; }
        else if (r.kind == 4) { out->table_rev_ms += ms; out->table_rev_launches += 1; out->table_rev_bytes += r.work; }
        else if (r.kind == 5) { out->emd_ms += ms; out->emd_launches += 1; out->emd_pairs += r.work; }
        else { out->phase2_ms += ms; out->phase2_launches += 1; out->phase2_bytes += r.work; out->phase2_gather_bytes += r.work2; }
    }
    ctx->prof.clear();
    out->emd_abandoned = ctx->prof_abandoned;
    return LCRWMD_OK;
}

const char* lcrwmd_last_error(const lcrwmd_ctx* ctx) { return ctx ? ctx->err : "context is NULL"; }

lcrwmd_status lcrwmd_set_options(lcrwmd_ctx* ctx, const lcrwmd_options* opt)
{
    if (!ctx) return LCRWMD_EINVAL;
    if (!opt) return fail(ctx, LCRWMD_EINVAL, "options are NULL");
    if ((opt->validate != 0 && opt->validate != 1) ||
        (opt->compute != LCRWMD_F32 && opt->compute != LCRWMD_BF16 && opt->compute != LCRWMD_BF16X3) ||
        opt->max_query_batch < 0 || opt->max_db_batch < 0 || opt->dedup < 0 || opt->dedup > 2)
        return fail(ctx, LCRWMD_EINVAL, "option out of range");
    ctx->opt = *opt;
    return LCRWMD_OK;
}

lcrwmd_status lcrwmd_get_options(const lcrwmd_ctx* ctx, lcrwmd_options* opt)
{
    if (!ctx || !opt) return LCRWMD_EINVAL;
    *opt = ctx->opt;
    return LCRWMD_OK;
}

lcrwmd_status lcrwmd_workspace_bytes(lcrwmd_ctx* ctx, int64_t v, int64_t m, int64_t n, int64_t nnz_db, int64_t q,
                                     int64_t nnz_q, lcrwmd_dtype emb_dtype, int k, size_t* out_bytes)
{
    if (!ctx) return LCRWMD_EINVAL;
    if (!out_bytes) return fail(ctx, LCRWMD_EINVAL, "out_bytes is NULL");
    if (v <= 0 || m <= 0 || n < 0 || nnz_db < 0 || q < 0 || nnz_q < 0 || k < 0)
        return fail(ctx, LCRWMD_EINVAL, "negative size");
    const bool asks_bf16 = emb_dtype == LCRWMD_BF16 || ctx->opt.compute == LCRWMD_BF16;
    const int bf16 = m > 300 ? 0 : asks_bf16 ? 1 : ctx->opt.compute == LCRWMD_BF16X3 ? 2 : 0;     // see prec_mode
    const bool widened = m > 300 && asks_bf16;
    int64_t qr = q > 0 ? q : 1;                                  // queries per range: all of them when they fit
    if (ctx->opt.dedup == 1 && qr > table_max_queries()) qr = table_max_queries();
    int64_t nb = n < kDbBatch ? n : kDbBatch;
    if (ctx->opt.max_db_batch > 0 && nb > ctx->opt.max_db_batch) nb = ctx->opt.max_db_batch;
    if (nb < 1) nb = 1;
    const int64_t vq = v < nnz_q ? v : nnz_q, ve_max = v < nnz_db ? v : nnz_db;
    const int64_t ldz = round_up(qr, 4);
    const bool padded = bf16 == 0 && m <= kPadM && m >= kPadFromM;
    const size_t fixed = rwmd_fixed_bytes(v, (int32_t)m, nnz_q, nnz_db, bf16, padded, widened);
    const size_t zfull = (size_t)ve_max * (size_t)ldz * 4 + 256;                       // first-phase minima of a range
    const size_t tile = (size_t)nb * (size_t)ldz * 4 + 256;                            // a block's tile (lcrwmd_rwmd_reduce)
    const size_t f = token_plan_bytes(qr, nnz_q) + close_bits_bytes(qr, ve_max);
    const size_t r = rev_batch_bytes(vq, nb, nnz_db) + tile + close_bits_bytes(nb, vq);
    size_t region = f > r ? f : r;
    // room for the word-pair table at its upper bound (distinct words <= stored entries); when the library picks the
    // form, only where its cost model picks the table at those bounds and the table then fits the device (a large
    // vocabulary against thousands of queries would otherwise ask for a table of terabytes that no range ever builds)
    if (ctx->opt.dedup) {
        const size_t t = (size_t)ve_max * (size_t)(round_up(vq, 32) + 32 * ((vq + 255) / 256)) * 4 + (size_t)(ve_max + 256) * 8 +
                         table_bucket_bytes(vq, qr, nnz_q) + (size_t)n * (size_t)ldz * 4 + 2 * tile + 8192;
        const bool wanted = ctx->opt.dedup == 1 ||
                            (qr <= table_max_queries() && table_form_is_faster(bf16, (int32_t)m, ve_max, vq, n, nnz_db, qr, nnz_q) &&
                             fixed + zfull + t <= ctx->device_bytes / 4 * 3);
        if (wanted && t > region) region = t;
    }
    size_t total = fixed + zfull + region + 4096;
    // lcrwmd_rwmd_reduce: the running lists, a block's list and its partial lists, the column sums' scratch
    total += 6 * ((size_t)qr * (size_t)(k > 0 ? k : 1) * 4 + 256) + topk_bytes(nb, qr, k > 0 ? k : 1) + col_sums_bytes(qr) + 2048;
    // the stand-alone first phase needs norms, the optional bf16 copy, one token plan (of either set) and, for the
    // queries, the map of close pairs (without room for the map the kernel's results are scanned instead)
    size_t p1 = emb_prep_bytes(v, (int32_t)m, bf16, padded, widened) + token_plan_bytes(q > n ? q : n, nnz_q > nnz_db ? nnz_q : nnz_db) +
                close_bits_bytes(q, v) + 4096;
    *out_bytes = total > p1 ? total : p1;
    return LCRWMD_OK;
}

lcrwmd_status lcrwmd_phase1_mindist(lcrwmd_ctx* ctx, const lcrwmd_emb* E, const lcrwmd_csr* queries, float* Z,
                                    int64_t ldz, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    ST_TRY(check_emb(ctx, E));
    ST_TRY(check_csr(ctx, queries, "queries", false));
    if (queries->cols != E->v) return fail(ctx, LCRWMD_EINVAL, "queries.cols must equal E.v");
    if (!Z) return fail(ctx, LCRWMD_EINVAL, "Z is NULL");
    if (ldz < queries->rows) return fail(ctx, LCRWMD_EINVAL, "ldz < queries.rows");
    if (queries->rows == 0) return LCRWMD_OK;
    ST_TRY(check_ws(ctx, ws, ws_bytes));
    if (queries->nnz + 7 * queries->rows >= kMaxTokens)
        return fail(ctx, LCRWMD_EUNSUPPORTED, "too many tokens for one pass; split the queries");
    HIP_TRY(hipSetDevice(ctx->device));
    Bump b(ws, ws_bytes);
    if (ctx->opt.validate) {
        int32_t* st = b.take_n<int32_t>(64);
        if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small");
        lcrwmd_csr tmp = *queries;
        tmp.val = nullptr;
        ST_TRY(validate_on_device(ctx, &tmp, "queries", st, s));
    }
    EmbPrep ep;
    ST_TRY(prepare_emb(ctx, E, b, ep, s));
    TokenPlan tp;
    carve_token_plan(b, tp, queries->rows, queries->nnz, plan_tiles((E->v + kTileVocab - 1) / kTileVocab, ep.bf16), -1,
                     plan_group(ep), plan_chunk_tiles(ep));
    if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small: need about %zu bytes",
                           emb_prep_bytes(E->v, (int32_t)E->m, ep.mode, wants_padded_copy(E), wants_widened_copy(ctx, E)) +
                               token_plan_bytes(queries->rows, queries->nnz));
    uint64_t* bits = take_close_bits(b, queries->rows, E->v);
    return run_phase1(ctx, ep, (int32_t)E->m, nullptr, E->v, 0, nullptr, queries->row_ptr, queries->col_idx,
                      queries->nnz, tp, Z, ldz, s, false, bits);
}

lcrwmd_status lcrwmd_phase2_spmm(lcrwmd_ctx* ctx, const lcrwmd_csr* X, const float* Z, int64_t ldz, int64_t ncols,
                                 float* D, int64_t ldd, int combine, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    ST_TRY(check_csr(ctx, X, "X", true));
    if (ncols < 0) return fail(ctx, LCRWMD_EINVAL, "ncols < 0");
    if (combine < 0 || combine > 2) return fail(ctx, LCRWMD_EINVAL, "combine must be 0, 1 or 2");
    if (X->rows == 0 || ncols == 0) return LCRWMD_OK;
    if (!Z || !D) return fail(ctx, LCRWMD_EINVAL, "Z or D is NULL");
    if (ldz < ncols) return fail(ctx, LCRWMD_EINVAL, "ldz < ncols");
    if (ldd < (combine == 2 ? X->rows : ncols)) return fail(ctx, LCRWMD_EINVAL, "ldd smaller than a row of D");
    HIP_TRY(hipSetDevice(ctx->device));
    return run_spmm(ctx, X->row_ptr, X->col_idx, X->val, X->rows, X->nnz, X->cols, Z, ldz, ncols, D, ldd, combine, s);
}

lcrwmd_status lcrwmd_rwmd(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database,
                          const lcrwmd_emb* E, float* D, int64_t ldd, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    ST_TRY(check_rwmd_args(ctx, queries, database, E));
    if (queries->rows == 0 || database->rows == 0) return LCRWMD_OK;
    if (!D) return fail(ctx, LCRWMD_EINVAL, "D is NULL");
    if (ldd < queries->rows) return fail(ctx, LCRWMD_EINVAL, "ldd < queries.rows");
    ST_TRY(check_ws(ctx, ws, ws_bytes));
    HIP_TRY(hipSetDevice(ctx->device));
    HostPtr rq, rdb;
    ST_TRY(fetch_rows_and_validate(ctx, queries, database, rq, rdb, ws, ws_bytes, s));
    ctx->forms_ran = 0;
    return rwmd_ranges(ctx, queries, rq.p, database, rdb.p, E, D, ldd, queries->rows, ws, ws_bytes, s);
}

lcrwmd_status lcrwmd_topk(lcrwmd_ctx* ctx, const float* D, int64_t n, int64_t q, int64_t ldd, int k, int32_t* R_idx,
                          float* R_dist, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    if (n < 0 || q < 0) return fail(ctx, LCRWMD_EINVAL, "negative size");
    if (q == 0) return LCRWMD_OK;
    if (!D || !R_idx || !R_dist) return fail(ctx, LCRWMD_EINVAL, "D, R_idx or R_dist is NULL");
    if (ldd < q) return fail(ctx, LCRWMD_EINVAL, "ldd < q");
    if (k < 1 || k > n) return fail(ctx, LCRWMD_EINVAL, "k must be in [1, n]");
    if (k > kMaxTopK) return fail(ctx, LCRWMD_EUNSUPPORTED, "k > %d is not supported", kMaxTopK);
    if (n > 0x7fffffffLL) return fail(ctx, LCRWMD_EUNSUPPORTED, "n exceeds int32 row indices");
    if (ws && ((uintptr_t)ws & 255) != 0) return fail(ctx, LCRWMD_EWORKSPACE, "the workspace must be 256-byte aligned");
    HIP_TRY(hipSetDevice(ctx->device));
    HIP_TRY(launch_topk(D, n, q, ldd, k, R_idx, R_dist, ws, ws ? ws_bytes : 0, s));
    return LCRWMD_OK;
}

lcrwmd_status lcrwmd_topk_noalloc(lcrwmd_ctx* ctx, const float* D, int64_t n, int64_t q, int64_t ldd, int k,
                                  int32_t* R_idx, float* R_dist, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    if (n < 0 || q < 0) return fail(ctx, LCRWMD_EINVAL, "negative size");
    if (q == 0) return LCRWMD_OK;
    if (!D || !R_idx || !R_dist) return fail(ctx, LCRWMD_EINVAL, "D, R_idx or R_dist is NULL");
    if (ldd < q) return fail(ctx, LCRWMD_EINVAL, "ldd < q");
    if (k < 1 || k > n) return fail(ctx, LCRWMD_EINVAL, "k must be in [1, n]");
    if (k > kMaxTopK) return fail(ctx, LCRWMD_EUNSUPPORTED, "k > %d is not supported", kMaxTopK);
    if (n > 0x7fffffffLL) return fail(ctx, LCRWMD_EUNSUPPORTED, "n exceeds int32 row indices");
    const size_t need = topk_bytes(n, q, k);
    if (need > topk_static_bytes())
        return fail(ctx, LCRWMD_EWORKSPACE, "the partial lists of this problem take %zu bytes, the built-in scratch holds %zu: "
                    "use lcrwmd_topk with a workspace", need, topk_static_bytes());
    void* scratch = topk_static_ptr(ctx->device);
    if (!scratch) return fail(ctx, LCRWMD_EHIP, "the scratch array of device %d was not found at lcrwmd_create", ctx->device);
    HIP_TRY(hipSetDevice(ctx->device));
    // every slot of the partial lists that the merge reads is written by the launch before it: nothing to clear
    HIP_TRY(launch_topk(D, n, q, ldd, k, R_idx, R_dist, scratch, need, s));
    return LCRWMD_OK;
}

}  // extern "C"

namespace {

// Sink of lcrwmd_rwmd_reduce: a running top-k per query (two lists that take turns) and running column sums.
struct ReduceSink : TileSink {
    lcrwmd_ctx* ctx = nullptr;
    int k = 0;
    int64_t q = 0;
    float* run_d[2] = {nullptr, nullptr};
    int32_t* run_i[2] = {nullptr, nullptr};
    float* blk_d = nullptr;
    int32_t* blk_i = nullptr;
    void* tk = nullptr;
    size_t tkb = 0;
    double* sums = nullptr;      // the caller's, already offset to this range's first query
    double* part = nullptr;
    int cur = 0;
    bool any = false;

    lcrwmd_status consume(int64_t i0, int64_t i1, const float* tile, int64_t ldt, hipStream_t s) override
    {
        if (k > 0) {
            // slots a block cannot fill read FLT_MAX; values that the k rows of the list so far already beat are skipped
            HIP_TRY(launch_topk(tile, i1 - i0, q, ldt, k, blk_i, blk_d, tk, tkb, s, any ? run_d[cur] : nullptr));
            HIP_TRY(launch_topk_merge2(run_d[cur], run_i[cur], any, blk_d, blk_i, i0, q, k, run_d[cur ^ 1], run_i[cur ^ 1], s));
            cur ^= 1;
        }
        if (sums) HIP_TRY(launch_col_sums(tile, i1 - i0, q, ldt, part, !any, sums, s));
        any = true;
        return LCRWMD_OK;
    }
};

// Sink of lcrwmd_rwmd_self.  A tile holds the distances of histograms [i0, i1) (rows) to the batch [j0, j1) (columns).
// Columns: as in ReduceSink, except that a column's list starts from what earlier batches already found for that
// histogram.  Rows beyond the batch: the same distances belong to those histograms' own lists and sums (the bound is
// symmetric), which are updated in place - no later batch computes these pairs again.
struct SelfSink : ReduceSink {
    int64_t j0 = 0, j1 = 0;
    int32_t* R_idx = nullptr;        // n x k, all histograms
    float* R_dist = nullptr;
    double* all_sums = nullptr;      // n, or null

    lcrwmd_status consume(int64_t i0, int64_t i1, const float* tile, int64_t ldt, hipStream_t s) override
    {
        ST_TRY(ReduceSink::consume(i0, i1, tile, ldt, s));
        const int64_t r0 = i0 > j1 ? i0 : j1;          // rows of the batch itself are columns too: nothing to mirror
        if (r0 < i1)
            HIP_TRY(launch_topk_rows(tile + (r0 - i0) * ldt, i1 - r0, q, ldt, k, j0, k > 0 ? R_dist + r0 * k : nullptr,
                                     k > 0 ? R_idx + r0 * k : nullptr, all_sums ? all_sums + r0 : nullptr, s));
        return LCRWMD_OK;
    }
};

}  // namespace

extern "C" {

lcrwmd_status lcrwmd_rwmd_reduce(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database,
                                 const lcrwmd_emb* E, int k, int32_t* R_idx, float* R_dist, double* col_sum,
                                 void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    ST_TRY(check_rwmd_args(ctx, queries, database, E));
    const int64_t n = database->rows, q = queries->rows;
    if (k < 0) return fail(ctx, LCRWMD_EINVAL, "k < 0");
    if (k == 0 && !col_sum) return fail(ctx, LCRWMD_EINVAL, "nothing asked for: k == 0 and col_sum is NULL");
    if (q == 0) return LCRWMD_OK;
    if (k > 0 && (!R_idx || !R_dist)) return fail(ctx, LCRWMD_EINVAL, "R_idx or R_dist is NULL");
    if (k > n) return fail(ctx, LCRWMD_EINVAL, "k must be in [1, n]");
    if (k > kMaxTopK) return fail(ctx, LCRWMD_EUNSUPPORTED, "k > %d is not supported", kMaxTopK);
    if (n > 0x7fffffffLL) return fail(ctx, LCRWMD_EUNSUPPORTED, "n exceeds int32 row indices");
    ST_TRY(check_ws(ctx, ws, ws_bytes));
    HIP_TRY(hipSetDevice(ctx->device));
    HostPtr rq, rdb;
    ST_TRY(fetch_rows_and_validate(ctx, queries, database, rq, rdb, ws, ws_bytes, s));
    ctx->forms_ran = 0;
    if (n == 0) return LCRWMD_OK;

    // Ranges of queries: all of them when their first-phase minima fit the workspace, otherwise fewer at a time.
    int64_t qr = q;
    if (ctx->opt.dedup == 1 && qr > table_max_queries()) qr = table_max_queries();
    int64_t nb = n < kDbBatch ? n : kDbBatch;
    if (ctx->opt.max_db_batch > 0 && nb > ctx->opt.max_db_batch) nb = ctx->opt.max_db_batch;
    for (int64_t j0 = 0; j0 < q;) {
        const int64_t j1 = j0 + qr < q ? j0 + qr : q, nq = j1 - j0;
        Bump b(ws, ws_bytes);
        ReduceSink sink;
        sink.ctx = ctx;
        sink.k = k;
        sink.q = nq;
        if (k > 0) {
            for (int t = 0; t < 2; ++t) {
                sink.run_d[t] = b.take_n<float>((size_t)nq * k);
                sink.run_i[t] = b.take_n<int32_t>((size_t)nq * k);
            }
            sink.blk_d = b.take_n<float>((size_t)nq * k);
            sink.blk_i = b.take_n<int32_t>((size_t)nq * k);
            sink.tkb = topk_bytes(nb, nq, k) + 512;
            sink.tk = b.take(sink.tkb);
        }
        if (col_sum) {
            sink.sums = col_sum + j0;
            sink.part = (double*)b.take(col_sums_bytes(nq));
        }
        bool shrink = !b.ok;
        lcrwmd_status st = LCRWMD_EWORKSPACE;
        if (b.ok) {
            const size_t off = (b.used + 255) & ~(size_t)255;
            st = off < ws_bytes ? rwmd_core(ctx, queries, rq.p, j0, j1, database, rdb.p, E, nullptr, 0, &sink, (char*)ws + off,
                                            ws_bytes - off, s, &shrink)
                                : LCRWMD_EWORKSPACE;
            if (off >= ws_bytes) shrink = true;
        }
        if (st == LCRWMD_EWORKSPACE && shrink && qr > 1) { qr = (qr + 1) / 2; continue; }     // nothing of this range was written
        if (st == LCRWMD_EWORKSPACE && !b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for the lists of one query");
        if (st != LCRWMD_OK) return st;
        if (k > 0) {
            HIP_TRY(hipMemcpyAsync(R_dist + j0 * k, sink.run_d[sink.cur], sizeof(float) * (size_t)nq * k, hipMemcpyDeviceToDevice, s));
            HIP_TRY(hipMemcpyAsync(R_idx + j0 * k, sink.run_i[sink.cur], sizeof(int32_t) * (size_t)nq * k, hipMemcpyDeviceToDevice, s));
        }
        j0 = j1;
    }
    return LCRWMD_OK;
}

lcrwmd_status lcrwmd_rwmd_topk(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database,
                               const lcrwmd_emb* E, int k, int32_t* R_idx, float* R_dist, void* ws, size_t ws_bytes,
                               void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    if (k < 1) return fail(ctx, LCRWMD_EINVAL, "k must be in [1, n]");
    return lcrwmd_rwmd_reduce(ctx, queries, database, E, k, R_idx, R_dist, nullptr, ws, ws_bytes, hip_stream);
}

lcrwmd_status lcrwmd_rwmd_self(lcrwmd_ctx* ctx, const lcrwmd_csr* docs, const lcrwmd_emb* E, int64_t batch, int k,
                               int32_t* R_idx, float* R_dist, double* dist_sum, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    ST_TRY(check_rwmd_args(ctx, docs, docs, E));
    const int64_t n = docs->rows;
    if (batch < 0) return fail(ctx, LCRWMD_EINVAL, "batch < 0");
    if (k < 0) return fail(ctx, LCRWMD_EINVAL, "k < 0");
    if (k == 0 && !dist_sum) return fail(ctx, LCRWMD_EINVAL, "nothing asked for: k == 0 and dist_sum is NULL");
    if (n == 0) return LCRWMD_OK;
    if (k > 0 && (!R_idx || !R_dist)) return fail(ctx, LCRWMD_EINVAL, "R_idx or R_dist is NULL");
    if (k > n) return fail(ctx, LCRWMD_EINVAL, "k must be in [1, n]");
    if (k > kMaxTopK) return fail(ctx, LCRWMD_EUNSUPPORTED, "k > %d is not supported", kMaxTopK);
    if (n > 0x7fffffffLL) return fail(ctx, LCRWMD_EUNSUPPORTED, "n exceeds int32 row indices");
    ST_TRY(check_ws(ctx, ws, ws_bytes));
    HIP_TRY(hipSetDevice(ctx->device));
    HostPtr rd, again;
    ST_TRY(fetch_rows_and_validate(ctx, docs, docs, rd, again, ws, ws_bytes, s));
    ctx->forms_ran = 0;
    const int64_t batch_cap = ctx->opt.dedup == 1 ? table_max_queries() : n;
    if (batch == 0) {
        // the largest power of two up to 65,536 whose workspace figure fits: larger batches share more of their words,
        // so the swapped first phase - rows of Z' = distinct words of a batch - does less work in total
        for (batch = 65536; batch > 1; batch /= 2) {
            const int64_t bb = batch < n ? batch : n;
            int64_t most = 0;
            for (int64_t a = 0; a < n; a += bb) {
                const int64_t e = rd.p[a + bb < n ? a + bb : n] - rd.p[a];
                if (e > most) most = e;
            }
            size_t need = 0;
            if (bb <= batch_cap && lcrwmd_workspace_bytes(ctx, E->v, E->m, n, docs->nnz, bb, most, E->dtype, k, &need) == LCRWMD_OK &&
                need <= ws_bytes)
                break;
        }
    }
    if (batch > n) batch = n;
    if (batch > batch_cap) batch = batch_cap;
    int64_t nb = n < kDbBatch ? n : kDbBatch;
    if (ctx->opt.max_db_batch > 0 && nb > ctx->opt.max_db_batch) nb = ctx->opt.max_db_batch;

    // every list empty, every sum zero
    if (k > 0) {
        HIP_TRY(launch_fill_i32(reinterpret_cast<int32_t*>(R_dist), n * k, 0x7f7fffff, s));     // FLT_MAX
        HIP_TRY(launch_fill_i32(R_idx, n * k, 0x7fffffff, s));
    }
    if (dist_sum) HIP_TRY(launch_fill_i32(reinterpret_cast<int32_t*>(dist_sum), 2 * n, 0, s));

    for (int64_t j0 = 0; j0 < n; j0 += batch) {
        const int64_t j1 = j0 + batch < n ? j0 + batch : n, nq = j1 - j0;
        Bump b(ws, ws_bytes);
        SelfSink sink;
        sink.ctx = ctx;
        sink.k = k;
        sink.q = nq;
        sink.j0 = j0;
        sink.j1 = j1;
        sink.R_idx = R_idx;
        sink.R_dist = R_dist;
        sink.all_sums = dist_sum;
        if (k > 0) {
            for (int t = 0; t < 2; ++t) {
                sink.run_d[t] = b.take_n<float>((size_t)nq * k);
                sink.run_i[t] = b.take_n<int32_t>((size_t)nq * k);
            }
            sink.blk_d = b.take_n<float>((size_t)nq * k);
            sink.blk_i = b.take_n<int32_t>((size_t)nq * k);
            sink.tkb = topk_bytes(nb, nq, k) + 512;
            sink.tk = b.take(sink.tkb);
        }
        if (dist_sum) {
            sink.sums = dist_sum + j0;
            sink.part = (double*)b.take(col_sums_bytes(nq));
        }
        const size_t off = (b.used + 255) & ~(size_t)255;
        if (!b.ok || off >= ws_bytes) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for the lists of a batch of %lld", (long long)nq);
        if (k > 0) {
            // the batch's lists so far: what the rows of earlier batches' tiles put there
            HIP_TRY(hipMemcpyAsync(sink.run_d[0], R_dist + j0 * k, sizeof(float) * (size_t)nq * k, hipMemcpyDeviceToDevice, s));
            HIP_TRY(hipMemcpyAsync(sink.run_i[0], R_idx + j0 * k, sizeof(int32_t) * (size_t)nq * k, hipMemcpyDeviceToDevice, s));
        }
        sink.any = true;                    // lists and sums continue, they do not start
        bool shrink = false;
        lcrwmd_status st = rwmd_core(ctx, docs, rd.p, j0, j1, docs, rd.p, E, nullptr, 0, &sink, (char*)ws + off, ws_bytes - off, s,
                                     &shrink, /*db_row0=*/j0);
        if (st == LCRWMD_EWORKSPACE)
            return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for batches of %lld histograms: size it with "
                        "lcrwmd_workspace_bytes for q = batch, or pass a smaller batch", (long long)batch);
        if (st != LCRWMD_OK) return st;
        if (k > 0) {
            HIP_TRY(hipMemcpyAsync(R_dist + j0 * k, sink.run_d[sink.cur], sizeof(float) * (size_t)nq * k, hipMemcpyDeviceToDevice, s));
            HIP_TRY(hipMemcpyAsync(R_idx + j0 * k, sink.run_i[sink.cur], sizeof(int32_t) * (size_t)nq * k, hipMemcpyDeviceToDevice, s));
        }
    }
    return LCRWMD_OK;
}

int lcrwmd_forms_ran(const lcrwmd_ctx* ctx) { return ctx ? ctx->forms_ran : 0; }

lcrwmd_status lcrwmd_probe_gather(lcrwmd_ctx* ctx, int64_t segments, int floats_per_lane, void* ws, size_t ws_bytes,
                                  double* tbytes_per_s, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    if (!tbytes_per_s) return fail(ctx, LCRWMD_EINVAL, "the output pointer is NULL");
    if (segments < 1 || segments > ((int64_t)1 << 24) || (segments & (segments - 1)) != 0)
        return fail(ctx, LCRWMD_EINVAL, "segments must be a power of two in [1, 2^24]");
    if (floats_per_lane != 1 && floats_per_lane != 2 && floats_per_lane != 4)
        return fail(ctx, LCRWMD_EINVAL, "floats_per_lane must be 1, 2 or 4");
    ST_TRY(check_ws(ctx, ws, ws_bytes));
    const size_t table = (size_t)segments * 4096 * 4;
    if (ws_bytes < table + 256) return fail(ctx, LCRWMD_EWORKSPACE, "the probe needs %zu bytes", table + 256);
    HIP_TRY(hipSetDevice(ctx->device));
    float* T = (float*)ws;
    float* out = (float*)((char*)ws + table);
    HIP_TRY(launch_fill_i32((int32_t*)ws, (int64_t)(table / 4) + 1, 0, s));
    const int blocks = ctx->num_cu * 8, iters = 400;
    double bytes = 0.0;
    HIP_TRY(launch_probe_gather(T, segments, floats_per_lane, blocks, iters / 4, out, &bytes, s));     // warm-up: caches and clock
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(ctx, LCRWMD_EHIP, "hipEventCreate failed"); }
    float ms = 0.f;
    hipError_t e = hipEventRecord(e0, s);
    if (e == hipSuccess) e = launch_probe_gather(T, segments, floats_per_lane, blocks, iters, out, &bytes, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return fail(ctx, LCRWMD_EHIP, "probe failed: %s", hipGetErrorString(e));
    *tbytes_per_s = bytes / (ms * 1e-3) / 1e12;
    return LCRWMD_OK;
}

lcrwmd_status lcrwmd_probe_mfma(lcrwmd_ctx* ctx, lcrwmd_dtype dtype, int random_data, int a_from_lds, double seconds,
                                void* ws, size_t ws_bytes, double* tflops, double* shader_mhz, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    if (dtype != LCRWMD_F32 && dtype != LCRWMD_BF16) return fail(ctx, LCRWMD_EINVAL, "dtype must be LCRWMD_F32 or LCRWMD_BF16");
    if (!tflops || !shader_mhz) return fail(ctx, LCRWMD_EINVAL, "an output pointer is NULL");
    if (!(seconds > 0.0) || seconds > 10.0) return fail(ctx, LCRWMD_EINVAL, "seconds must be in (0, 10]");
    ST_TRY(check_ws(ctx, ws, ws_bytes));
    if (ws_bytes < probe_bytes(ctx->num_cu)) return fail(ctx, LCRWMD_EWORKSPACE, "the probe needs %zu bytes", probe_bytes(ctx->num_cu));
    HIP_TRY(hipSetDevice(ctx->device));
    // iterations for about `seconds` at the spec-sheet rate (32 MFMAs of 8 / 16 passes per iteration and wavefront, two
    // workgroups of four wavefronts per CU share the four matrix pipes of a CU)
    const double clocks_per_iter = 32.0 * (dtype == LCRWMD_BF16 ? 32 : 64) * 2;
    int iters = (int)(seconds * 2.4e9 / clocks_per_iter);
    if (iters < 1000) iters = 1000;
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(ctx, LCRWMD_EHIP, "hipEventCreate failed"); }
    double flops = 0.0;
    long long* clk = nullptr;
    long long h[2] = {0, 1};
    float ms = 0.f;
    hipError_t e = hipEventRecord(e0, s);
    if (e == hipSuccess) e = launch_probe_mfma(dtype == LCRWMD_BF16, random_data != 0, a_from_lds != 0, iters, ctx->num_cu, ws, &flops, &clk, s);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) e = hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return fail(ctx, LCRWMD_EHIP, "probe failed: %s", hipGetErrorString(e));
    *tflops = flops / ((double)ms * 1e-3) / 1e12;
    *shader_mhz = (double)h[0] / (double)(h[1] > 0 ? h[1] : 1) * 100.0;      // the wall-clock counter ticks at 100 MHz
    return LCRWMD_OK;
}

// Quadratic-complexity RWMD (Sec. III "Solving the RWMD problem", Sec. V first GPU mapping): every database
// histogram against every query through its own T matrices, nothing shared between histograms.
namespace {
size_t quadratic_block_bytes(int64_t nb, int64_t nnz_b, int64_t q, int64_t nnz_q)
{
    const size_t a = token_plan_bytes(q, nnz_q) + (size_t)nnz_b * (size_t)round_up(q, 4) * 4 + close_bits_bytes(q, nnz_b) + 512;      // row minima
    const size_t b = token_plan_bytes(nb, nnz_b) + (size_t)nnz_q * (size_t)round_up(nb, 4) * 4 + close_bits_bytes(nb, nnz_q) + 512;  // column minima
    return a > b ? a : b;
}
}  // namespace

lcrwmd_status lcrwmd_rwmd_quadratic_workspace_bytes(lcrwmd_ctx* ctx, int64_t v, int64_t m, int64_t n, int64_t nnz_db,
                                                    int64_t q, int64_t nnz_q, lcrwmd_dtype emb_dtype, size_t* out_bytes)
{
    if (!ctx) return LCRWMD_EINVAL;
    if (!out_bytes) return fail(ctx, LCRWMD_EINVAL, "out_bytes is NULL");
    if (v <= 0 || m <= 0 || n < 0 || nnz_db < 0 || q < 0 || nnz_q < 0) return fail(ctx, LCRWMD_EINVAL, "negative size");
    const bool asks_bf16 = emb_dtype == LCRWMD_BF16 || ctx->opt.compute == LCRWMD_BF16;
    const int mode = m > 300 ? 0 : asks_bf16 ? 1 : ctx->opt.compute == LCRWMD_BF16X3 ? 2 : 0;
    const bool padded = mode == 0 && m <= kPadM && m >= kPadFromM;
    // blocks of database rows: about 2^20 stored entries each, never more rows than the swapped pass of lcrwmd_rwmd takes
    int64_t nb = n < 4096 ? (n > 0 ? n : 1) : 4096;
    const int64_t nnz_b = n > 0 ? (nnz_db / n + 1) * nb * 2 : 1;
    *out_bytes = emb_prep_bytes(v, (int32_t)m, mode, padded, m > 300 && asks_bf16) + ((size_t)(nnz_b > nnz_q ? nnz_b : nnz_q) * 4 + 256) +
                 quadratic_block_bytes(nb, nnz_b < nnz_db ? nnz_b : nnz_db, q > 0 ? q : 1, nnz_q) + 8192;
    return LCRWMD_OK;
}

lcrwmd_status lcrwmd_rwmd_quadratic(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database,
                                    const lcrwmd_emb* E, float* D, int64_t ldd, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    ST_TRY(check_rwmd_args(ctx, queries, database, E));
    const int64_t n = database->rows, q = queries->rows, nnz_q = queries->nnz;
    if (q == 0 || n == 0) return LCRWMD_OK;
    if (!D) return fail(ctx, LCRWMD_EINVAL, "D is NULL");
    if (ldd < q) return fail(ctx, LCRWMD_EINVAL, "ldd < queries.rows");
    ST_TRY(check_ws(ctx, ws, ws_bytes));
    HIP_TRY(hipSetDevice(ctx->device));
    HostPtr rq, rdb;
    ST_TRY(fetch_rows_and_validate(ctx, queries, database, rq, rdb, ws, ws_bytes, s));
    if (nnz_q + 7 * q >= kMaxTokens) return fail(ctx, LCRWMD_EUNSUPPORTED, "too many query words for one pass; split the queries");
    const int32_t m = (int32_t)E->m;
    Bump b(ws, ws_bytes);
    EmbPrep ep;
    ST_TRY(prepare_emb(ctx, E, b, ep, s));
    const int grp = plan_group(ep), chunk_tiles = plan_chunk_tiles(ep);

    // Blocks of database rows whose two matrices of minima fit the workspace.
    const size_t fixed_off = (b.used + 255) & ~(size_t)255;
    int64_t nb = n < 4096 ? n : 4096;
    int64_t iota_len = 0;
    for (;;) {
        const int64_t tok = max_tokens_per_batch(rdb.p, n, nb);
        iota_len = tok > nnz_q ? tok : nnz_q;
        const size_t need = fixed_off + (size_t)iota_len * 4 + 512 + quadratic_block_bytes(nb, tok, q, nnz_q) + 1024;
        if (tok + 7 * nb < kMaxTokens && need <= ws_bytes) break;
        if (nb == 1) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for one database row against all queries");
        nb = (nb + 1) / 2;
    }
    int32_t* iota = b.take_n<int32_t>((size_t)iota_len);          // column ids of a stacked T matrix's rows: 0, 1, 2, ...
    if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "internal: index array does not fit");
    HIP_TRY(launch_iota_i32(iota, iota_len, s));
    const size_t region_off = (b.used + 255) & ~(size_t)255;
    const size_t region = ws_bytes - region_off;

    for (int64_t i0 = 0; i0 < n; i0 += nb) {
        const int64_t i1 = i0 + nb < n ? i0 + nb : n;
        const int64_t t0 = rdb.p[i0], nnz_b = rdb.p[i1] - t0;
        float* Db = D + i0 * ldd;
        {   // C = T1 o T2,j for all j at once (Sec. III): row minima of every stacked database word against each query,
            // then the dot products with the database weights: D12 = F1 . Z1
            Bump bb((char*)ws + region_off, region);
            TokenPlan tp;
            carve_token_plan(bb, tp, q, nnz_q, plan_tiles((nnz_b + kTileVocab - 1) / kTileVocab, ep.bf16), padded_tokens(rq.p, 0, q, grp), grp,
                             chunk_tiles);
            const int64_t ldz = round_up(q, 4);
            float* Z1 = bb.take_n<float>((size_t)nnz_b * ldz);
            if (!bb.ok) return fail(ctx, LCRWMD_EWORKSPACE, "internal: row minima do not fit");
            uint64_t* bits = take_close_bits(bb, q, nnz_b);
            ST_TRY(run_phase1(ctx, ep, m, database->col_idx + t0, nnz_b, 1, nullptr, queries->row_ptr, queries->col_idx, nnz_q, tp, Z1,
                              ldz, s, false, bits));
            // rows of the block in their stacked order: entry p of the block reads row p - t0 of Z1
            ST_TRY(run_spmm(ctx, database->row_ptr + i0, iota - t0, database->val, i1 - i0, nnz_b, nnz_b, Z1, ldz, q, Db, ldd, 0, s));
        }
        {   // column minima: every query word against each database histogram of the block, D21 = F2 . Z2, and the maximum
            Bump bb((char*)ws + region_off, region);
            TokenPlan tp;
            carve_token_plan(bb, tp, i1 - i0, nnz_b, plan_tiles((nnz_q + kTileVocab - 1) / kTileVocab, ep.bf16),
                             padded_tokens(rdb.p, i0, i1, grp), grp, chunk_tiles);
            const int64_t ldz = round_up(i1 - i0, 4);
            float* Z2 = bb.take_n<float>((size_t)nnz_q * ldz);
            if (!bb.ok) return fail(ctx, LCRWMD_EWORKSPACE, "internal: column minima do not fit");
            uint64_t* bits = take_close_bits(bb, i1 - i0, nnz_q);
            ST_TRY(run_phase1(ctx, ep, m, queries->col_idx, nnz_q, 1, nullptr, database->row_ptr + i0, database->col_idx, nnz_b, tp, Z2,
                              ldz, s, /*swapped=*/true, bits));
            ST_TRY(run_spmm(ctx, queries->row_ptr, iota, queries->val, q, nnz_q, nnz_q, Z2, ldz, i1 - i0, Db, ldd, 2, s));
        }
    }
    return LCRWMD_OK;
}

// ------------------------------------------------------------------------------------------------ exact WMD, WCD, pruning

lcrwmd_status lcrwmd_wcd(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database, const lcrwmd_emb* E,
                         float* D, int64_t ldd, void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    ST_TRY(check_rwmd_args(ctx, queries, database, E));
    const int64_t n = database->rows, q = queries->rows;
    if (n == 0 || q == 0) return LCRWMD_OK;
    if (!D) return fail(ctx, LCRWMD_EINVAL, "D is NULL");
    if (ldd < q) return fail(ctx, LCRWMD_EINVAL, "ldd < queries.rows");
    ST_TRY(check_ws(ctx, ws, ws_bytes));
    HIP_TRY(hipSetDevice(ctx->device));
    Bump b(ws, ws_bytes);
    if (ctx->opt.validate) {
        int32_t* st = b.take_n<int32_t>(64);
        if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small");
        ST_TRY(validate_on_device(ctx, queries, "queries", st, s));
        ST_TRY(validate_on_device(ctx, database, "database", st, s));
    }
    const int64_t ldc = round_up(E->m, 4);
    float* C1 = b.take_n<float>((size_t)n * ldc);
    float* C2 = b.take_n<float>((size_t)q * ldc);
    if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for the centroids: need %zu bytes",
                           (size_t)(n + q) * ldc * 4 + 1024);
    HIP_TRY(launch_centroids(*E, *database, C1, ldc, s));
    HIP_TRY(launch_centroids(*E, *queries, C2, ldc, s));
    HIP_TRY(launch_centroid_dist(C1, n, C2, q, ldc, (int32_t)E->m, D, ldd, s));
    return LCRWMD_OK;
}

lcrwmd_status lcrwmd_wmd_pairs_workspace_bytes(lcrwmd_ctx* ctx, int64_t max_h_db, int64_t max_h_q, int64_t pairs_in_flight,
                                               size_t* out_bytes)
{
    if (!ctx) return LCRWMD_EINVAL;
    if (!out_bytes) return fail(ctx, LCRWMD_EINVAL, "out_bytes is NULL");
    if (max_h_db <= 0 || max_h_q <= 0) return fail(ctx, LCRWMD_EINVAL, "sizes must be positive");
    if (pairs_in_flight <= 0) pairs_in_flight = emd_preferred_slots(ctx->num_cu, max_h_db, max_h_q);
    *out_bytes = emd_pair_bytes(max_h_db, max_h_q) * (size_t)pairs_in_flight + 1024;
    return LCRWMD_OK;
}

}  // extern "C"

namespace {

int64_t longest_row(const int64_t* rp, int64_t rows)
{
    int64_t mx = 0;
    for (int64_t r = 0; r < rows; ++r)
        if (rp[r + 1] - rp[r] > mx) mx = rp[r + 1] - rp[r];
    return mx;
}

// WMD of `count` listed pairs into out; the wavefronts that solve them share `slabs`.  counters: [0] failures
// (accumulated), [2] the work queue's position, [3] pairs abandoned above their limit (accumulated).
// limit (or nullptr): pair (i, j) may be abandoned, its output set to FLT_MAX, once its distance is known to exceed
// limit[j - limit_j0].
lcrwmd_status run_wmd_list(lcrwmd_ctx* ctx, const lcrwmd_csr* Q, const lcrwmd_csr* DB, const lcrwmd_emb* E,
                           const int32_t* pair_db, const int32_t* pair_q, int64_t count, int64_t h1max, int64_t h2max,
                           void* slabs, size_t slab_bytes, float* out, int32_t* flags, int32_t* counters, hipStream_t s,
                           const float* limit = nullptr, int32_t limit_j0 = 0)
{
    if (count <= 0) return LCRWMD_OK;
    if (count > 0x7fffffffLL) return fail(ctx, LCRWMD_EUNSUPPORTED, "more than 2^31 pairs in one list");
    int64_t slots = (int64_t)(slab_bytes / emd_pair_bytes(h1max, h2max));
    const int64_t pref = emd_preferred_slots(ctx->num_cu, h1max, h2max);
    if (slots > pref) slots = pref;
    if (slots < 1) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for one transport problem (%zu bytes)",
                               emd_pair_bytes(h1max, h2max));
    ProfScope ps(ctx, s, 5, (double)count);
    HIP_TRY(launch_emd(*E, *DB, *Q, pair_db, pair_q, count, h1max, h2max, slabs, slots, counters + 2, out, flags, counters,
                       limit, limit_j0, counters + 3, s));
    return LCRWMD_OK;
}

}  // namespace

extern "C" {

lcrwmd_status lcrwmd_wmd_pairs(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database, const lcrwmd_emb* E,
                               const int32_t* pair_db, const int32_t* pair_q, int64_t npairs, float* out, int32_t* flags,
                               void* ws, size_t ws_bytes, void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    ST_TRY(check_rwmd_args(ctx, queries, database, E));
    if (npairs < 0) return fail(ctx, LCRWMD_EINVAL, "npairs < 0");
    if (npairs == 0) return LCRWMD_OK;
    if (!pair_db || !pair_q || !out) return fail(ctx, LCRWMD_EINVAL, "pair_db, pair_q or out is NULL");
    if (queries->rows == 0 || database->rows == 0) return fail(ctx, LCRWMD_EINVAL, "pairs listed but a set is empty");
    ST_TRY(check_ws(ctx, ws, ws_bytes));
    HIP_TRY(hipSetDevice(ctx->device));
    HostPtr rq, rdb;
    ST_TRY(fetch_rows_and_validate(ctx, queries, database, rq, rdb, ws, ws_bytes, s));
    const int64_t h1max = longest_row(rdb.p, database->rows), h2max = longest_row(rq.p, queries->rows);
    if (!emd_supported(h1max, h2max))
        return fail(ctx, LCRWMD_EUNSUPPORTED, "histograms of %lld + %lld words exceed the solver's per-word state in LDS",
                    (long long)h1max, (long long)h2max);
    Bump b(ws, ws_bytes);
    int32_t* counters = b.take_n<int32_t>(64);
    if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small");
    HIP_TRY(launch_fill_i32(counters, 4, 0, s));
    if (ctx->opt.validate) {
        HIP_TRY(launch_check_pairs(pair_db, pair_q, npairs, database->rows, queries->rows, counters + 1, s));
        int32_t bad = 0;
        HIP_TRY(hipMemcpyAsync(&bad, counters + 1, sizeof(bad), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        if (bad) return fail(ctx, LCRWMD_EINVAL, "a listed pair is outside [0, n) x [0, q)");
    }
    const size_t off = (b.used + 255) & ~(size_t)255;
    ST_TRY(run_wmd_list(ctx, queries, database, E, pair_db, pair_q, npairs, h1max, h2max, (char*)ws + off, ws_bytes - off, out,
                        flags, counters, s));
    if (!flags) {
        int32_t failed = 0;
        HIP_TRY(hipMemcpyAsync(&failed, counters, sizeof(failed), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        if (failed) return fail(ctx, LCRWMD_ENOCONVERGE, "%d transport problems ran out of their augmentation budget", failed);
    }
    return LCRWMD_OK;
}

lcrwmd_status lcrwmd_wmd_topk_workspace_bytes(lcrwmd_ctx* ctx, int64_t v, int64_t m, int64_t n, int64_t nnz_db, int64_t q,
                                              int64_t nnz_q, lcrwmd_dtype emb_dtype, int k, int64_t max_h_db,
                                              int64_t max_h_q, size_t* out_bytes)
{
    if (!ctx) return LCRWMD_EINVAL;
    if (!out_bytes) return fail(ctx, LCRWMD_EINVAL, "out_bytes is NULL");
    if (k < 1 || max_h_db <= 0 || max_h_q <= 0) return fail(ctx, LCRWMD_EINVAL, "k and the histogram sizes must be positive");
    size_t base = 0;
    ST_TRY(lcrwmd_workspace_bytes(ctx, v, m, n, nnz_db, q, nnz_q, emb_dtype, kMaxTopK < n ? kMaxTopK : (k > (int)n ? k : (int)n), &base));
    int64_t qb = q < 2048 ? q : 2048;
    if (ctx->opt.max_query_batch > 0 && qb > ctx->opt.max_query_batch) qb = ctx->opt.max_query_batch;
    // per-query arrays, lists for a quarter of all pairs of a batch, one transport problem per resident wavefront
    const size_t lists = (size_t)qb * (size_t)kMaxTopK * 24 + (size_t)qb * 32 + (size_t)n * (size_t)qb / 4 * 12;
    const size_t slabs = emd_pair_bytes(max_h_db, max_h_q) * (size_t)emd_preferred_slots(ctx->num_cu, max_h_db, max_h_q);
    // the n x qb tile of bounds the pruning reads, and the scratch of the top-k over it
    const size_t tile = (size_t)n * (size_t)round_up(qb, 4) * 4 + topk_bytes(n, qb, kMaxTopK) + 1024;
    *out_bytes = base + tile + lists + slabs + 16384;
    return LCRWMD_OK;
}

lcrwmd_status lcrwmd_wmd_topk(lcrwmd_ctx* ctx, const lcrwmd_csr* queries, const lcrwmd_csr* database, const lcrwmd_emb* E,
                              int k, int32_t* R_idx, float* R_dist, int64_t* evaluated, void* ws, size_t ws_bytes,
                              void* hip_stream)
{
    if (!ctx) return LCRWMD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    ST_TRY(check_rwmd_args(ctx, queries, database, E));
    const int64_t n = database->rows, q = queries->rows;
    if (q == 0) return LCRWMD_OK;
    if (!R_idx || !R_dist) return fail(ctx, LCRWMD_EINVAL, "R_idx or R_dist is NULL");
    if (k < 1 || k > n) return fail(ctx, LCRWMD_EINVAL, "k must be in [1, n]");
    if (k > kMaxTopK) return fail(ctx, LCRWMD_EUNSUPPORTED, "k > %d is not supported", kMaxTopK);
    if (n > (int64_t)65535 * 256) return fail(ctx, LCRWMD_EUNSUPPORTED, "more than 16.7 million database rows");
    if (E->dtype == LCRWMD_F32 && ctx->opt.compute == LCRWMD_BF16)
        return fail(ctx, LCRWMD_EUNSUPPORTED, "pruning needs a true lower bound: fp32 E with bf16 compute is refused");
    ST_TRY(check_ws(ctx, ws, ws_bytes));
    HIP_TRY(hipSetDevice(ctx->device));
    HostPtr rq, rdb;
    ST_TRY(fetch_rows_and_validate(ctx, queries, database, rq, rdb, ws, ws_bytes, s));
    const int64_t h1max = longest_row(rdb.p, n), h2max = longest_row(rq.p, q);
    if (!emd_supported(h1max, h2max))
        return fail(ctx, LCRWMD_EUNSUPPORTED, "histograms of %lld + %lld words exceed the solver's per-word state in LDS",
                    (long long)h1max, (long long)h2max);
    const size_t pair_bytes = emd_pair_bytes(h1max, h2max);
    const int mode = prec_mode(ctx, E);

    // Query batches.  Front of the workspace: the n x qb tile of RWMD bounds and the per-query arrays; the rest
    // serves first the RWMD passes and then the candidate lists and the transport problems.
    int64_t qb = q < 2048 ? q : 2048;
    if (ctx->opt.max_query_batch > 0 && qb > ctx->opt.max_query_batch) qb = ctx->opt.max_query_batch;
    auto front_bytes = [&](int64_t b) {
        return (size_t)n * (size_t)round_up(b, 4) * 4 + topk_bytes(n, b, kMaxTopK) + (size_t)b * (size_t)kMaxTopK * 24 +
               (size_t)b * 32 + 8192;
    };
    for (;;) {
        const int64_t ve_max = E->v < database->nnz ? E->v : database->nnz, vq_max = E->v < queries->nnz ? E->v : queries->nnz;
        const size_t rwmd_need = rwmd_fixed_bytes(E->v, (int32_t)E->m, queries->nnz, database->nnz, mode,
                                                     mode == 0 && wants_padded_copy(E), wants_widened_copy(ctx, E)) +
                                 (size_t)ve_max * (size_t)round_up(qb, 4) * 4 + token_plan_bytes(qb, max_tokens_per_batch(rq.p, q, qb)) +
                                 rev_batch_bytes(vq_max, 1, max_tokens_per_batch(rdb.p, n, 1)) + 8192;
        const size_t wmd_need = (size_t)qb * (size_t)kMaxTopK * 16 + pair_bytes * 2 + 8192;   // first-round lists, a problem in flight
        if (front_bytes(qb) + (rwmd_need > wmd_need ? rwmd_need : wmd_need) <= ws_bytes) break;
        if (qb == 1) return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for a one-query batch");
        qb = (qb + 1) / 2;
    }
    std::vector<int64_t> hoff;
    try {
        hoff.resize((size_t)qb + 1);
    } catch (const std::bad_alloc&) {
        return fail(ctx, LCRWMD_EINVAL, "out of host memory");
    }
    int32_t failed_total = 0;
    for (int64_t j0 = 0; j0 < q; j0 += qb) {
        const int64_t j1 = j0 + qb < q ? j0 + qb : q, nq = j1 - j0;
        Bump b(ws, ws_bytes);
        const int64_t ldt = round_up(nq, 4);
        // First round: the k1 >= k nearest by RWMD per query, solved to the end.  The paper takes k1 = k; while the
        // batch's k * nq transport problems do not fill the device, a larger k1 costs no time and gives a lower cut-off
        // (the k-th smallest of k1 distances instead of the largest of k), hence fewer survivors.  Nothing is lost: any
        // k evaluated distances bound the k-th best from above.
        // Second round, when the first one already fills the device with k per query: the next nearest up to 64 per
        // query against that cut-off (abandoned as soon as they pass it, like survivors, so they cost little), after
        // which the cut-off is the k-th smallest of all evaluated so far.  (With fewer queries the wider first round
        // does the same without a launch of its own, which would be bound by the latency of its few full solves.)
        const int kmax = n < kMaxTopK ? (int)n : kMaxTopK;
        int k1 = (int)(emd_preferred_slots(ctx->num_cu, h1max, h2max) / nq);
        if (k1 > kmax) k1 = kmax;
        const bool full_device = k1 <= k;
        if (k1 < k) k1 = k;
        const int kx = full_device ? kmax : k1;                  // candidates taken off the top of the bounds
        const int k2 = kx - k1;
        float* tile = b.take_n<float>((size_t)n * ldt);
        const size_t tkb = topk_bytes(n, nq, kx) + 512;
        void* tk = b.take(tkb);
        int32_t* R0 = b.take_n<int32_t>((size_t)nq * kx);
        float* R0d = b.take_n<float>((size_t)nq * kx);
        int32_t* p0_db = b.take_n<int32_t>((size_t)nq * kx);
        int32_t* p0_q = b.take_n<int32_t>((size_t)nq * kx);
        float* wmd0 = b.take_n<float>((size_t)nq * kx);
        float* wmd1 = wmd0 + (size_t)nq * k1;                    // second round: k2 per query
        float* cut = b.take_n<float>((size_t)nq);
        int32_t* cnt = b.take_n<int32_t>((size_t)nq);
        int64_t* off = b.take_n<int64_t>((size_t)nq + 1);
        int64_t* cursor = b.take_n<int64_t>((size_t)nq);
        int32_t* counters = b.take_n<int32_t>(64);
        if (!b.ok) return fail(ctx, LCRWMD_EWORKSPACE, "internal: query batch does not fit");
        const size_t rest_off = (b.used + 255) & ~(size_t)255;
        char* rest = (char*)ws + rest_off;
        const size_t rest_bytes = ws_bytes - rest_off;

        // RWMD to every database histogram, the kx nearest by RWMD (Sec. III)
        ST_TRY(rwmd_core(ctx, queries, rq.p, j0, j1, database, rdb.p, E, tile, ldt, nullptr, rest, rest_bytes, s, nullptr));
        HIP_TRY(launch_topk(tile, n, nq, ldt, kx, R0, R0d, tk, tkb, s));
        // WMD to the first k1 of those; the k-th smallest of them is the cut-off
        HIP_TRY(launch_fill_i32(counters, 4, 0, s));
        HIP_TRY(launch_first_pairs(R0, nq, kx, 0, k1, (int32_t)j0, tile, ldt, p0_db, p0_q, s));
        ST_TRY(run_wmd_list(ctx, queries, database, E, p0_db, p0_q, nq * k1, h1max, h2max, rest, rest_bytes, wmd0, nullptr,
                            counters, s));
        HIP_TRY(launch_cutoff(wmd0, k1, wmd1, 0, nq, k, 1e-5f, cut, s));
        if (k2 > 0) {
            int32_t* p1_db = p0_db + (size_t)nq * k1;
            int32_t* p1_q = p0_q + (size_t)nq * k1;
            HIP_TRY(launch_first_pairs(R0, nq, kx, k1, kx, (int32_t)j0, tile, ldt, p1_db, p1_q, s));
            ST_TRY(run_wmd_list(ctx, queries, database, E, p1_db, p1_q, nq * k2, h1max, h2max, rest, rest_bytes, wmd1, nullptr,
                                counters, s, cut, (int32_t)j0));
            HIP_TRY(launch_cutoff(wmd0, k1, wmd1, k2, nq, k, 1e-5f, cut, s));
        }
        // survivors: RWMD below the cut-off
        HIP_TRY(launch_count_below(tile, n, nq, ldt, cut, cnt, off, s));
        HIP_TRY(hipMemcpyAsync(hoff.data(), off, sizeof(int64_t) * ((size_t)nq + 1), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        if (evaluated)
            for (int64_t j = 0; j < nq; ++j) evaluated[j0 + j] = kx + hoff[j + 1] - hoff[j];
        // Lists hold 12 bytes per survivor; they share `rest` with the transport problems in flight.
        // The transport problems get all the room they can use when the batch's lists fit beside it in one piece,
        // half of the rest otherwise.
        size_t slab_part = pair_bytes * (size_t)emd_preferred_slots(ctx->num_cu, h1max, h2max);
        const size_t lists_all = (size_t)hoff[nq] * 12 + 8192;
        if (slab_part + lists_all > rest_bytes && slab_part > rest_bytes / 2) slab_part = rest_bytes / 2;
        if (slab_part < pair_bytes) slab_part = pair_bytes;
        slab_part = (slab_part + 255) / 256 * 256;
        if (slab_part + 4096 > rest_bytes)
            return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small for one transport problem");
        const int64_t list_cap = (int64_t)((rest_bytes - slab_part - 2048) / 12);
        for (int64_t ja = 0; ja < nq;) {
            int64_t jb = ja;
            while (jb < nq && hoff[jb + 1] - hoff[ja] <= list_cap) ++jb;
            if (jb == ja)
                return fail(ctx, LCRWMD_EWORKSPACE, "workspace too small: query %lld alone has %lld survivors (%lld fit)",
                            (long long)(j0 + ja), (long long)(hoff[ja + 1] - hoff[ja]), (long long)list_cap);
            const int64_t total = hoff[jb] - hoff[ja];
            Bump lb(rest + slab_part, rest_bytes - slab_part);
            int32_t* l_db = lb.take_n<int32_t>((size_t)total + 1);
            int32_t* l_q = lb.take_n<int32_t>((size_t)total + 1);
            float* l_d = lb.take_n<float>((size_t)total + 1);
            if (!lb.ok) return fail(ctx, LCRWMD_EWORKSPACE, "internal: survivor lists do not fit");
            HIP_TRY(launch_fill_below(tile, n, ja, jb, ldt, cut, off, cursor, (int32_t)j0, l_db, l_q, s));
            // a survivor is dropped as soon as the solver's lower bound on its distance passes the cut-off
            ST_TRY(run_wmd_list(ctx, queries, database, E, l_db, l_q, total, h1max, h2max, rest, slab_part, l_d, nullptr, counters, s,
                                cut, (int32_t)j0));
            HIP_TRY(launch_select_lists(R0, wmd0, k1, wmd1, k2, k, off, ja, jb, l_db, l_d, R_idx + j0 * k, R_dist + j0 * k, s));
            ja = jb;
        }
        int32_t hc[4] = {0, 0, 0, 0};
        HIP_TRY(hipMemcpyAsync(hc, counters, sizeof(hc), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        failed_total += hc[0];
        if (ctx->profiling) ctx->prof_abandoned += (double)hc[3];
    }
    if (failed_total)
        return fail(ctx, LCRWMD_ENOCONVERGE, "%d transport problems ran out of their augmentation budget", failed_total);
    return LCRWMD_OK;
}

}  // extern "C"
