// Internal declarations shared by the translation units of the LC-RWMD library.
// Host-side launch wrappers live next to their kernels; api.hip only orchestrates.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/lcrwmd.h"

struct lcrwmd_prof_rec {
    hipEvent_t start, stop;
    int kind;              // 1: first-phase kernel, 2: second-phase kernel, 3/4: table passes, 5: transport solver
    double work, work2;
};

struct lcrwmd_ctx {
    int device;
    int num_cu;
    size_t device_bytes;              // the device's total memory
    lcrwmd_options opt;
    char err[512];
    bool profiling;
    int forms_ran = 0;                // bit 0: the per-entry form ran in the last bound call, bit 1: the table form
    double prof_abandoned = 0.0;      // lcrwmd_wmd_topk: survivors whose solve stopped above the cut-off, while profiling
    std::vector<lcrwmd_prof_rec> prof;
};

namespace lcrwmd {

// ---------------------------------------------------------------------------------------------
// Padded token list of a batch of histograms (the stacked T matrix of Sec. IV, many-to-many
// form, kept as word ids instead of gathered vectors).  Every histogram ("segment") is padded to
// a multiple of `group` tokens by repeating its last word, which leaves every minimum unchanged and
// makes each group of consecutive tokens belong to exactly one segment.  In the 32x32 MFMA
// accumulator a lane holds runs of 4 consecutive rows, and a lane and its partner 32 lanes up hold
// 8 consecutive rows between them: kernels work on groups of 8, or of 4 where the shorter padding pays.
// ---------------------------------------------------------------------------------------------
constexpr int kGroup = 8;          // largest group size (bounds the padding)
constexpr int kGroupMin = 4;       // smallest group size (bounds the number of groups)
constexpr int kTileTokens = 128;   // token rows per tile of the first-phase kernel
constexpr int kTileVocab = 128;    // vocabulary columns per workgroup of the first-phase kernel

struct TokenPlan {
    // sizes known on the host
    int64_t nseg;          // histograms in the batch
    int64_t tok_bound;     // upper bound on padded tokens: stored entries + 7 per histogram
    int64_t tok_alloc;     // allocated padded tokens (bound rounded up to a tile, plus one tile)
    int32_t chunk_tokens;  // target padded tokens per chunk (multiple of kTileTokens)
    int32_t nchunks;       // upper bound on chunks
    int32_t group;         // tokens per group: 4 or 8
    // device arrays (carved from the workspace)
    int32_t* pofs;         // [nseg + 1] padded token offset of each segment
    int32_t* tok_ids;      // [tok_alloc] word id per padded token (0 beyond the end)
    float* tok_hn;         // [tok_alloc] -0.5 * |E[word]|^2 per padded token
    int32_t* grp_seg;      // [tok_alloc / group] segment of each group, -1 beyond the end
    int32_t* chunk_seg;    // [nchunks + 1] first segment of each chunk
};

size_t token_plan_bytes(int64_t nseg, int64_t nnz_batch);

struct Bump {   // carves 256-byte aligned pieces from the caller's workspace
    char* base;
    size_t size, used;
    bool ok;
    Bump(void* p, size_t n) : base((char*)p), size(n), used(0), ok(true) {}
    void* take(size_t bytes)
    {
        size_t a = (used + 255) & ~(size_t)255;
        if (!ok || a + bytes > size) { ok = false; return nullptr; }
        used = a + bytes;
        return base + a;
    }
    template <class T> T* take_n(size_t count) { return (T*)take(count * sizeof(T)); }
};

// padded_exact: the exact padded token count when the caller knows the row lengths (else -1: the bound is used,
// and the last chunks may turn out empty)
// max_chunk_tiles: upper limit on a chunk's length in tiles of kTileTokens.  Kernels whose workgroups own one chunk
// and reload the vocabulary operand for it want long chunks (64); the kernel that walks runs of chunks without
// reloading balances its load in units of chunks and wants short ones (kShortChunkTiles).
constexpr int kLongChunkTiles = 64, kShortChunkTiles = 8;
bool carve_token_plan(Bump& b, TokenPlan& tp, int64_t nseg, int64_t nnz_batch, int64_t nvoc_tiles,
                      int64_t padded_exact = -1, int group = kGroup, int max_chunk_tiles = kLongChunkTiles);

// Operand description of one first-phase launch.
struct Phase1Args {
    const void* E;            // fp32: caller's E.  bf16: packed copy made by pack_bf16
    int64_t ld;               // row pitch of E in elements
    int64_t erows = -1;       // rows of the matrix E points at (all of them, not only those this pass touches); the tile
                              // kernels address rows with 32-bit offsets and need to know that they suffice
    int32_t m;                // embedding dimension
    const float* normE;       // [v] squared norms by word id
    const int32_t* voc_rows;  // word ids that form the vocabulary of this pass, or nullptr = 0..nvoc-1
    int64_t nvoc;
    int z_by_position;        // 1: Z row = position in voc_rows; 0: Z row = word id
    float* Z;
    int64_t ldz;
    int32_t num_cu = 256;     // compute units of the device (the bf16 kernel launches one workgroup per CU)
    uint64_t* close_bits = nullptr;   // optional: map of the entries that came out close (see close_bits_pitch); written
                                      // by the tile kernels only - launch_phase1_* report whether it was
};

// prep.hip
hipError_t launch_fill_i32(int32_t* p, int64_t n, int32_t value, hipStream_t s);
hipError_t launch_iota_i32(int32_t* p, int64_t n, hipStream_t s);      // p[i] = i
hipError_t launch_row_norms_f32(const float* E, int64_t v, int32_t m, int64_t ld, float* normE, hipStream_t s);
// fp32 copy (pitch m) of E's values as bf16 numbers: bf16 storage widened, fp32 storage rounded to nearest even
hipError_t launch_widen_bf16(const void* E, lcrwmd_dtype dtype, int64_t v, int32_t m, int64_t ld, float* out, hipStream_t s);
// copy of E with `pitch` >= m floats per row (zeros beyond column m) and the squared norms
hipError_t launch_pack_f32(const float* E, int64_t v, int32_t m, int64_t ld, int32_t pitch, float* packed, float* normE,
                           hipStream_t s);
hipError_t launch_mark_words(const int32_t* col_idx, int64_t nnz, int32_t* flags, hipStream_t s);
// list[pos] = w and map[w] = pos for flagged words (map[w] = -1 otherwise); *count = number flagged
hipError_t launch_compact_words(const int32_t* flags, int64_t v, int32_t* list, int32_t* map, int32_t* count,
                                hipStream_t s);
hipError_t launch_remap_cols(const int32_t* col_idx, int64_t nnz, const int32_t* map, int32_t* out, hipStream_t s);
hipError_t launch_token_plan(const TokenPlan& tp, const int64_t* row_ptr_batch, const int32_t* col_idx,
                             const float* normE, hipStream_t s);
// Z[row(word) * ldz + seg] = 0 for every stored (seg, word) of the batch; row() through map when given
hipError_t launch_zero_matches(const int64_t* row_ptr_batch, const int32_t* col_idx, int64_t nseg,
                               const int32_t* map, float* Z, int64_t ldz, hipStream_t s, uint64_t* bits = nullptr,
                               int64_t pitch = 0, int slice_words = 0);
// Entries of Z (rows by position in voc_rows, or by word id when voc_rows is null) whose square is below a quarter of
// the word's squared norm are recomputed from coordinate differences over the histogram's words.  E: fp32 rows, or
// bf16 rows when `bf16`, pitch ld elements.  Runs after launch_zero_matches.
hipError_t launch_redo_close(const void* E, bool bf16, int64_t ld, int32_t m, const float* normE, const int32_t* voc_rows,
                             int64_t nvoc, const int64_t* row_ptr_batch, const int32_t* col_idx, int64_t nseg, float* Z,
                             int64_t ldz, hipStream_t s);
// The same from the contraction kernel's map of close pairs instead of a read of all of Z: bits[pitch * j + slice] has
// bit l set when entry (vocabulary position slice * slice_words + l % slice_words, histogram j) needs the second look.
hipError_t launch_redo_close_bits(const void* E, bool bf16, int64_t ld, int32_t m, const int32_t* voc_rows, int64_t nvoc,
                                  const int64_t* row_ptr_batch, const int32_t* col_idx, int64_t nseg, float* Z, int64_t ldz,
                                  const uint64_t* bits, int64_t pitch, int slice_words, hipStream_t s);
// status[0] = 0 ok, 2 bad csr, 3 empty doc (values of lcrwmd_status)
hipError_t launch_validate_csr(const lcrwmd_csr& X, int32_t* status, hipStream_t s);

// phase1_f32.hip
hipError_t launch_phase1_f32(const Phase1Args& a, const TokenPlan& tp, hipStream_t s);

// phase1_bf16.hip
bool bf16_supported(int32_t m);    // the register-resident vocabulary operand holds m + 4 <= 304 columns
size_t pack_bf16_bytes(int64_t v, int32_t m);
int32_t bf16_pitch(int32_t m);
hipError_t launch_pack_bf16(const void* E, lcrwmd_dtype dtype, int64_t v, int32_t m, int64_t ld, void* packed,
                            float* normE, hipStream_t s);
hipError_t launch_phase1_bf16(const Phase1Args& a, const TokenPlan& tp, hipStream_t s);

// phase1_tiles.hip: the direct-to-LDS tile kernel for both precisions
bool tiles_rows_addressable(int64_t rows, int64_t pitch_bytes);
bool tiles_f32_supported(const Phase1Args& a);
hipError_t launch_phase1_tiles_f32(const Phase1Args& a, const TokenPlan& tp, hipStream_t s);
hipError_t launch_phase1_tiles_bf16(const Phase1Args& a, const TokenPlan& tp, int num_cu, hipStream_t s);
hipError_t launch_phase1_tiles_x3(const Phase1Args& a, const TokenPlan& tp, hipStream_t s);
int phase1_group_x3();             // group size the split-bf16 kernel expects of its token plan
// Map of close pairs (Phase1Args::close_bits): vocabulary positions per 64-bit word, words per histogram; bytes for a batch
int close_bits_slice(int mode);
int64_t close_bits_pitch(int mode, int64_t nvoc);
inline size_t close_bits_bytes(int64_t nseg, int64_t nvoc) { return (size_t)nseg * (size_t)((nvoc + 255) / 256 * 8) * 8 + 256; }
// split-bf16 operand copy: 640 bf16 per row (304 hi values, 304 lo values, zeros)
size_t pack_x3_bytes(int64_t v);
int32_t x3_pitch();
hipError_t launch_pack_x3(const float* E, int64_t v, int32_t m, int64_t ld, void* packed, float* normE, hipStream_t s);
// mode: 0 fp32 rows, 1 packed bf16 rows, 2 split-bf16 rows
bool distance_table_supported(const Phase1Args& a, int mode);
hipError_t launch_distance_table(const Phase1Args& a, int mode, const int32_t* tok_ids, const float* tok_hn,
                                 int64_t ntok, hipStream_t s);
// table.hip: the two passes of the de-duplicated form over a word-pair table W (rows: distinct database words)
int64_t table_max_queries();
hipError_t launch_table_tokens(const int32_t* list_db, int64_t ve, const float* normE, int32_t* tok_ids, float* tok_hn,
                               int64_t count, hipStream_t s);
hipError_t launch_table_zero_same(const int32_t* list_q, int64_t vq, const int32_t* map_db, float* W, int64_t ldw,
                                  hipStream_t s);
// table entries of two different words that lie close (w^2 < |row word|^2 / 4) recomputed from coordinate differences
hipError_t launch_table_redo_close(const void* E, bool bf16, int64_t ld, int32_t m, const float* normE,
                                   const int32_t* list_db, int64_t ve, const int32_t* col_word, int64_t vc, float* W,
                                   int64_t ldw, hipStream_t s);
void table_strips(int64_t vq, int32_t* ws, int32_t* nstrip);
size_t table_bucket_bytes(int64_t vq, int64_t q, int64_t nnz_q);
hipError_t launch_table_spread(const int32_t* list_q, int64_t vq, const int32_t* pos_in, int64_t nnz, int32_t* col_word,
                               int32_t* pos_out, hipStream_t s);
hipError_t launch_table_buckets(const int64_t* q_rp, const int32_t* q_pos, const float* q_val, int64_t q, int64_t vq,
                                int32_t* cnt, int32_t* offs, int32_t* cursor, int32_t* bpos, float* bval, hipStream_t s);
hipError_t launch_table_fwd(const float* W, int64_t ldw, int64_t ve, int64_t vq, const int32_t* offs, const int32_t* bpos,
                            int64_t q, float* Z, int64_t ldz, hipStream_t s);
hipError_t launch_table_rev(const float* W, int64_t ldw, int64_t vq, const int64_t* db_rp, const int32_t* db_pos,
                            int64_t rows, const int32_t* offs, const int32_t* bpos, const float* bval, int64_t q,
                            float* D2, int64_t ld2, float* D, int64_t ldd, hipStream_t s);

// phase2.hip
// zrows: rows of Z (every col_idx is below it)
hipError_t launch_spmm(const int64_t* row_ptr, const int32_t* col_idx, const float* val, int64_t rows,
                       const float* Z, int64_t ldz, int64_t zrows, int64_t ncols, float* D, int64_t ldd, int combine,
                       hipStream_t s);

// topk.hip
constexpr int kMaxTopK = 64;
size_t topk_bytes(int64_t n, int64_t q, int k);
// bound (optional): q x k sorted lists of distances that earlier rows already reach; values not below a list's last
// entry are skipped (slots left unfilled read FLT_MAX / INT_MAX)
hipError_t launch_topk(const float* D, int64_t n, int64_t q, int64_t ldd, int k, int32_t* R_idx, float* R_dist,
                       void* ws, size_t ws_bytes, hipStream_t s, const float* bound = nullptr);
// out = the k smallest of list a (absolute row indices; ignored unless have_a) and list b (row indices relative to row0)
hipError_t launch_topk_merge2(const float* a_d, const int32_t* a_i, bool have_a, const float* b_d, const int32_t* b_i,
                              int64_t row0, int64_t q, int k, float* out_d, int32_t* out_i, hipStream_t s);
// sums[j] (+)= sum over the rows of tile[r][j] in fp64 (first: sums start at 0); part: col_sums_bytes(q) of scratch
size_t col_sums_bytes(int64_t q);
hipError_t launch_col_sums(const float* tile, int64_t rows, int64_t q, int64_t ldt, double* part, bool first, double* sums,
                           hipStream_t s);
// rows of a tile against the lists of their histograms (k nearest so far, in place) and their running sums: tile row
// r, column c is the distance of histogram row (R_dist + r * k) to histogram col_id0 + c
hipError_t launch_topk_rows(const float* tile, int64_t rows, int64_t q, int64_t ldt, int k, int64_t col_id0, float* R_dist,
                            int32_t* R_idx, double* row_sum, hipStream_t s);
// the file-scope device array behind lcrwmd_topk_noalloc: its size, the per-device address look-up (device current)
size_t topk_static_bytes();
hipError_t topk_static_init(int device);
void* topk_static_ptr(int device);

// probe.hip: bare MFMA loops (diagnostic)
size_t probe_bytes(int num_cu);
hipError_t launch_probe_gather(const float* T, int64_t rows, int width, int blocks, int iters, float* out, double* bytes,
                               hipStream_t s);
hipError_t launch_probe_mfma(bool bf16, bool random, bool a_from_lds, int iters, int num_cu, void* ws, double* flops,
                             long long** clk_dev, hipStream_t s);

// wmd.hip: transport problems (one wavefront each), centroid distances, pruning lists
size_t emd_pair_bytes(int64_t h1max, int64_t h2max);
bool emd_supported(int64_t h1max, int64_t h2max);
int64_t emd_preferred_slots(int num_cu, int64_t h1max, int64_t h2max);
hipError_t launch_emd(const lcrwmd_emb& E, const lcrwmd_csr& DB, const lcrwmd_csr& Q, const int32_t* pair_db,
                      const int32_t* pair_q, int64_t count, int64_t h1max, int64_t h2max, void* slabs, int64_t slots,
                      int32_t* next_pair, float* out, int32_t* flags, int32_t* fail_count, const float* limit,
                      int32_t limit_j0, int32_t* give_up_count, hipStream_t s);
hipError_t launch_check_pairs(const int32_t* pair_db, const int32_t* pair_q, int64_t npairs, int64_t n, int64_t q,
                              int32_t* status, hipStream_t s);
hipError_t launch_centroids(const lcrwmd_emb& E, const lcrwmd_csr& X, float* C, int64_t ldc, hipStream_t s);
hipError_t launch_centroid_dist(const float* C1, int64_t n, const float* C2, int64_t q, int64_t ldc, int32_t m, float* D,
                                int64_t ldd, hipStream_t s);
hipError_t launch_first_pairs(const int32_t* R0, int64_t q, int stride, int lo, int hi, int32_t j0, float* D, int64_t ldd,
                              int32_t* pair_db, int32_t* pair_q, hipStream_t s);
hipError_t launch_cutoff(const float* wa, int ka, const float* wb, int kb, int64_t q, int k, float slack, float* cut,
                         hipStream_t s);
hipError_t launch_count_below(const float* D, int64_t n, int64_t q, int64_t ldd, const float* cut, int32_t* cnt,
                              int64_t* off, hipStream_t s);
hipError_t launch_fill_below(const float* D, int64_t n, int64_t ja, int64_t jb, int64_t ldd, const float* cut,
                             const int64_t* off, int64_t* cursor, int32_t j0, int32_t* pair_db, int32_t* pair_q,
                             hipStream_t s);
hipError_t launch_select_lists(const int32_t* idx0, const float* da, int ka, const float* db, int kb, int k, const int64_t* off,
                               int64_t ja, int64_t jb, const int32_t* idx1, const float* d1, int32_t* R_idx, float* R_dist,
                               hipStream_t s);

}  // namespace lcrwmd
