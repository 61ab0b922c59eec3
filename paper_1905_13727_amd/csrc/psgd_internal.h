// Internal tables shared by the host planner and the device kernels.
// Plain structs only: they are copied byte-for-byte to the GPU.
#ifndef PSGD_INTERNAL_H
#define PSGD_INTERNAL_H

#include <stdint.h>
#include <string>
#include <vector>

#include "psgd.h"

namespace psgd {

constexpr int kWave = 64;          // gfx950 wavefront
constexpr int kBlock = 256;        // threads per workgroup in the streaming kernels (4 waves)
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kAlignElems = 64;    // every matrix starts on a multiple of this many elements
constexpr int kMaxVecPerLaneK1 = 2;  // column vectors a lane owns per row in the P = M Q kernel
constexpr int kMaxVecPerLaneK3 = 2;  // column vectors a lane owns in the Q = M^T P and decompress kernels
constexpr int kOrthoBlock = 256;   // threads of the single-workgroup Gram-Schmidt kernel
constexpr int kValuMaxRank = 8;    // ranks up to this run on the vector-ALU kernels
constexpr int kPanelFloats = 12288;  // n*r up to this: Gram-Schmidt by one workgroup with the panel in LDS (48 KB)
constexpr int kGramRows = 256;     // rows per workgroup of the Gram / apply kernels (Cholesky-QR over row blocks)
constexpr int kPreReduceParts = 16; // more partial-P slices than this: a reduction kernel runs before the orthogonalisation
constexpr int kOrthoMaxRows = 1024; // largest value of the tuning key ortho_rows: panels with more rows always take the multi-workgroup route
constexpr int kFlatTileElems = 1024;        // baselines: elements of a flattened matrix per workgroup of the elementwise sweep (one 16-byte access per
                                            // lane and array: the smallest slices were the fastest, 8192 -> 1024: 34.7 -> 28.7 us on the ResNet18 set)
constexpr int kFactorAlignElems = 4;        // P and Q of a matrix start at multiples of 4 floats (vector loads of factor rows)
constexpr int kHrGramTileRows = 128;       // matrix-core path: rows per workgroup of the mean-P / Gram / apply kernels
constexpr int64_t kHrMaxRows = 1 << 22;   // matrix-core path: tallest matrix (an n x 64 factor is addressed with 31-bit byte offsets)
constexpr int64_t kHrMaxCols = 1 << 20;   // matrix-core path: longest row (tiles of <= 256 rows are addressed with 31-bit byte offsets)
constexpr int64_t kStreamHintBytes = int64_t(320) << 20;   // update matrices of all workers above this (the 256 MB memory-side
                                                           // cache and a margin): the sweeps after the first treat M as a stream

// One matrix of the model.
struct MatDesc {
    int64_t off;        // element offset in the matrix region
    int64_t p_off;      // float offset in packed P
    int64_t q_off;      // float offset in packed Q
    int64_t ppart_off;  // float offset in the workspace: partial P, [W * n_cchunk][n][r]
    int64_t qpart_off;  // float offset in the workspace: partial Q, [W * n_rblock][m][r]
    int64_t gram_off;   // Cholesky-QR panels: offset (in doubles) of the Gram partials, [n_gblock][r*r]
    int32_t n, m, r;    // rows, columns, effective rank
    int32_t vec;        // elements per vector access along a row (4, 2 or 1)
    int32_t n_cchunk;   // column chunks of the P = M Q kernel (partials to sum)
    int32_t n_rblock;   // row blocks of the Q = M^T P kernel (partials to sum)
    int32_t tensor;     // index in the caller's shape list
    int32_t n_gblock;   // row blocks of the Gram / apply kernels; 0 = panel orthogonalised by one workgroup in LDS (k_ortho)
    int32_t pad_[2];
    int64_t chol_off;   // matrix-core path: offset (in doubles) of this matrix's Cholesky factor, r*r + r values
    int64_t kept_off;   // Random Block / Random K baselines: offset of this matrix's kept values (and indices) in their packed buffers
    int64_t kept;       // ... and their number, min((n + m) * rank, n * m)
};

// One workgroup's share of a streaming kernel.
struct Tile {
    int32_t mat;    // matrix index; -1: a slice of the vector region
    int32_t row0;   // first row (vector tiles: unused)
    int32_t nrows;  // rows
    int32_t vec0;   // first column vector (units of MatDesc::vec elements);
                    // vector tiles: first element / 4 is not assumed, see elem0 below
    int32_t nvec;   // column vectors
    int32_t part;   // which partial buffer slice this tile writes
    int64_t elem0;  // vector tiles and Q-reduce tiles: first element
    int64_t nelem;  // vector tiles and Q-reduce tiles: element count
};

// Resident path: one wavefront keeps one tile of M in registers through the whole step.
constexpr int kResRows = 32;         // most rows of a resident tile (registers: rows * vec floats per lane) ...
constexpr int res_rows_for_rank(int r) { return r <= 2 ? 32 : 24; }   // ... fewer when the rank needs the registers
constexpr int kResMinRows = 8;       // strips are not made thinner than this
constexpr int kResMaxN = 512;        // tallest matrix the single-wavefront Gram-Schmidt handles (8 rows per lane)
constexpr int kResMaxRank = 4;
constexpr int kResCUs = 256;         // MI355X compute units: the planner's provisional figure (it runs without a device); the
                                     // tiling is laid out again for the device's own count when the tables are uploaded
constexpr int kResBlocksPerCU = 2;   // 256-thread workgroups per compute unit (8 wavefronts, 2 per SIMD)
constexpr int kResTracePoints = 16;  // diagnostic timestamps per workgroup of the resident kernel

// One wavefront's share of the resident kernel.
struct RTile {
    int32_t mat;         // matrix index; -1: slice of the vector region; -2: idle slot
    int32_t row0, nrows; // strip of rows (nrows <= kResRows)
    int32_t vec0, nvec;  // column vectors (nvec <= 64)
    int32_t ppart;       // column-chunk index = slice of partial P this tile writes; the wavefront with
                         // ppart == 0 adds the chunks of its strip, the one that also has row0 == 0
                         // orthogonalises the matrix
    int32_t nstrips_mat; // strips of this matrix
    int32_t qrun_len;    // > 0: first of a run of consecutive wavefronts of the workgroup that hold strips of
                         // the same column chunk; it adds the run's sums in LDS and writes one partial Q
    int32_t qpart;       // slot of that partial; the run with qpart == 0 adds the chunk's partials
    int32_t nqparts;     // partial-Q slots of this column chunk
    int32_t cntq;        // running index of this column chunk over the model
    int32_t cnts;        // running index of this strip over the model
    int32_t pad_;
    int64_t elem0, nelem;  // vector tiles: slice of the vector region
};

struct Tuning {
    int64_t k1_rows = 0;    // rows per workgroup tile, P = M Q; 0: by the access width of the matrix (16 / 32 / 64; twice
                            // that for small sets)
    int64_t k1_nv = 2;      // column vectors per lane (<= kMaxVecPerLaneK1)
    int64_t k3_rows = 0;    // rows per workgroup tile, Q = M^T P; 0: 128, or 1024 for matrices >= 2048 x 2048
    int64_t k3_nv = 1;      // column vectors per lane (<= kMaxVecPerLaneK3)
    int64_t k4_rows = 0;    // rows per workgroup tile, decompress + residual; 0: 16 (32 for small sets)
    int64_t k4_nv = 1;
    int64_t hr_k3_rows = 2048;  // matrix-core Q = M^T P: rows per workgroup (four strips)
    int64_t hr_k4_rows = 0;     // matrix-core decompression: rows per workgroup (four strips of 16-row steps); 0 = by rank
    int64_t hr_k1_rows = 128;   // matrix-core P = M Q: rows per workgroup (multiple of 64, at most 256)
    int64_t hr_k1_cols = 2048;  // matrix-core P = M Q: columns per workgroup (multiple of 64); longer rows are split and their partial P summed
    int64_t stream_hints = -1;  // sweeps 2 and 3 of the streaming path: non-temporal loads of M and stores of the error
                                // memory (and temporal instead of non-temporal stores of Delta'); matrix-core path:
                                // non-temporal loads of M in sweep 2.
                                // -1: when M of all workers exceeds kStreamHintBytes; 0: never; 1: always
    int64_t gram_fused = 1; // Cholesky-QR panels: 1 = Gram matrices and factorisation in one launch when the device holds a matrix's
                            // row blocks at once; 0 = always the two launches; 2 = one launch whatever the device holds
                            // (diagnostic: the waits may time out, which psgd_plan_check then reports)
    int64_t gram_spin = 1 << 18;   // polls of one slot in that launch before a wait gives up
    int64_t ortho_rows = 0;        // panels of at most this many rows (and kPanelFloats values) are orthogonalised by one workgroup
                                   // with Gram-Schmidt in LDS (k_ortho), the others by Cholesky-QR over row blocks; 0: none (a
                                   // launch of its own for the short panels costs more than it saves: ResNet18-shaped set,
                                   // streaming, rank 2 / 4 / 8: 61.9 / 73.1 / 110.4 us with 1024, 59.6 / 67.0 / 100.9 us with 0)
    int64_t bf16_valu = -1; // bf16 gradients / output at rank <= 8: 1 = the streaming (vector-ALU) kernels, 0 = the matrix-core kernels,
                            // -1 = the matrix-core kernels at rank >= 4 on a set beyond the memory-side cache whose shapes they take
    int64_t resident = 1;   // 1: psgd_step keeps M on chip when the model fits; 0: always stream; 2: as 1 without the check
                            // against the device at upload (diagnostic, with res_max_blocks: lets a test see the waits give up)
    int64_t res_spin = 1 << 21;      // polls before a wait of the resident kernel gives up
    int64_t res_max_blocks = 0;      // 0: the device's capacity; else the most workgroups the resident tiling may use (diagnostic)
    int64_t res_rows = 0;   // 0: smallest strip height that fits; else forced strip height
    int64_t res_trace = 0;  // 1: the resident kernel records phase timestamps (diagnostic)
    int64_t xcd_order = -1;    // tile lists are ordered so that each accelerator die (own L2) works on one contiguous range of
                               // tiles: 1 = of the whole list; k >= 2 = of each group of consecutive matrices, a group being
                               // closed once it holds k tiles (a large matrix is then spread over all dies by itself); 0 = off;
                               // -1 = the planner's choice (groups sized by the worker count)
};

struct DeviceTables {
    MatDesc* mats = nullptr;
    Tile* tiles1 = nullptr;
    Tile* tiles3 = nullptr;
    Tile* tiles4 = nullptr;
    Tile* tiles4u = nullptr;   // decompression fused with the update: tiles of its own, or null (then tiles4)
    Tile* tilesq = nullptr;
    Tile* tiles_gram = nullptr;
    Tile* tilesp = nullptr;
    Tile* hr_tiles1 = nullptr;
    Tile* hr_tiles3 = nullptr;
    Tile* hr_tiles4 = nullptr;
    int64_t* flat_first = nullptr;         // baselines: per matrix the index of its first slice of kFlatTileElems elements
    int32_t* kept_slice_mat = nullptr;     // baselines: per slice of kBlock kept entries, its matrix ...
    int64_t* kept_slice_first = nullptr;   // ... and its first entry within that matrix
    int32_t* mat_tensor = nullptr;         // per matrix: index in the caller's tensor list
    int32_t* small_mats = nullptr;
    unsigned* gram_sync = nullptr;              // k_gram_chol: error word, epoch, finished-workgroup count
    unsigned long long* gram_mail = nullptr;    // k_gram_chol: the row blocks' Gram matrices as {value, epoch} slots
    MatDesc* res_mats = nullptr;
    RTile* res_tiles = nullptr;
    unsigned* res_sync = nullptr;  // error word, epoch, finished-workgroup count
    unsigned long long* res_mail = nullptr;  // mailbox of {value, epoch} slots
    unsigned long long* res_trace = nullptr;  // only with tuning res_trace = 1
    void* base = nullptr;   // the one allocation holding all of the above
};

}  // namespace psgd

struct psgd_plan {
    int32_t rank = 0;
    int32_t workers = 0;
    psgd_dtype grad_dtype = PSGD_F32;
    psgd_dtype out_dtype = PSGD_F32;
    psgd_sizes sizes{};
    std::vector<psgd_shape> shapes;
    std::vector<int64_t> tensor_flat_off;   // per tensor
    std::vector<int32_t> tensor_mat;        // per tensor: matrix index or -1
    std::vector<psgd::MatDesc> mats;
    std::vector<psgd::Tile> tiles1, tiles3, tiles4, tilesq;
    std::vector<psgd::Tile> tiles4u;        // third sweep when fused with the update, if its tiles differ (else empty)
    std::vector<psgd::Tile> tiles_gram;     // row blocks of the panels orthogonalised by Cholesky-QR
    std::vector<int64_t> flat_first;        // baselines (Appendix G): running count of the slices of the flattened matrices
    int64_t flat_tiles = 0;                 //   (n_matrices + 1 entries), their total, and the slices of the vector region
    int64_t flat_vec_tiles = 0;
    std::vector<int32_t> kept_slice_mat;    // baselines: slices of kBlock kept entries (matrix, first entry)
    std::vector<int64_t> kept_slice_first;
    std::vector<int32_t> mat_tensor;
    int64_t kept_slices = 0;
    std::vector<int32_t> small_mats;        // matrices orthogonalised by one workgroup (Gram-Schmidt in LDS)
    int64_t ws_gram_doubles = 0;            // workspace: Gram partials, after the float regions
    // matrix-core path (rank > 8, or bf16 gradients / output)
    bool hr = false;
    int32_t hr_nt = 1;                      // 16-wide rank tiles
    std::vector<psgd::Tile> hr_tiles1, hr_tiles3, hr_tiles4;
    int64_t ws_chol_doubles = 0;
    std::vector<psgd::Tile> tilesp;         // 64-element slices of the n x r panels (pre-reduction of partial P)
    bool p_pre_reduce = false;              // some matrix has more than kPreReduceParts partial-P slices
    bool stream_hints = false;              // see Tuning::stream_hints
    bool gram_fused = false;                // Cholesky-QR panels: one launch (k_gram_chol) instead of two (set at upload)
    int32_t max_n = 0;
    int64_t ws_ppart_floats = 0;            // workspace: partial P region (floats)
    int64_t ws_qpart_floats = 0;            // workspace: partial Q region, starts after partial P
    psgd::Tuning tuning;
    // resident path
    bool resident_ok = false;               // planner found a tiling that fits the chip
    int32_t res_strip_rows = 0;
    int32_t res_blocks = 0;
    int32_t res_vec_class = 0;
    std::vector<psgd::MatDesc> res_mats;    // same matrices, partial-sum layout of the resident tiling
    std::vector<psgd::RTile> res_tiles;     // res_blocks * 4 entries
    int32_t res_n_cntq = 0;                 // column-chunk arrival counters
    int32_t res_n_cnts = 0;                 // strip arrival counters
    int64_t res_ws_floats = 0;
    int64_t res_sync_words = 0;
    int64_t res_mail_slots = 0;             // 64-bit mailbox slots (plan-owned device memory)
    bool tables_built = false;
    bool uploaded = false;
    int device = -1;
    void* static_ws = nullptr;              // the library-owned workspace on that device (psgd_step_static)
    psgd::DeviceTables dev;
    std::string last_error;
    // per-kernel timing (benchmarks only)
    bool profiling = false;
    bool compress_marked = false;            // a compress call has recorded its events since profiling was switched on
    void* events[PSGD_N_KERNELS + 2] = {};   // hipEvent_t: before/after each kernel
    double kernel_ms[PSGD_N_KERNELS] = {};
    int64_t profiled_steps = 0;
};

namespace psgd {
// Algorithm 2's last two lines fused into the decompression: m <- lambda m + Delta', x <- x - gamma (Delta' + m),
// on buffers laid out like `out` (fp32); Delta' itself is then not stored.  mom == nullptr: plain decompression.
struct UpdateArgs {
    float* mom = nullptr;
    float* param = nullptr;
    float lr = 0.f;
    float lam = 0.f;
};
// host planner (psgd_plan.cpp)
psgd_status build_tables(psgd_plan* plan);
// lays the resident tiling out for a device that holds `max_blocks` workgroups at once (sets plan->resident_ok)
void build_resident(psgd_plan* plan, int64_t max_blocks);
// device side (psgd_kernels.hip)
psgd_status upload_tables(psgd_plan* plan);
void free_tables(psgd_plan* plan);
// add = false: one more subspace iteration on the update already held in err (grad is not read, err not written)
psgd_status launch_compress(psgd_plan* plan, const void* grad, float* err, float* q, float* p,
                            void* workspace, void* stream, bool add = true);
psgd_status launch_decompress(psgd_plan* plan, const float* p, const float* q, float* err,
                              const void* grad, void* out, void* workspace, void* stream,
                              const UpdateArgs& upd = UpdateArgs());
psgd_status set_profiling(psgd_plan* plan, bool enable);
psgd_status launch_q_reduce(psgd_plan* plan, float* ws, float* q, void* stream);
psgd_status finish_profiled_step(psgd_plan* plan);
psgd_status hr_compress(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* workspace,
                        void* stream, bool add);
psgd_status hr_decompress(psgd_plan* plan, const float* p, const float* q, float* err, const void* grad, void* out,
                          void* stream, const UpdateArgs& upd);
psgd_status launch_vector_mean(psgd_plan* plan, const void* grad, void* out, void* stream, const UpdateArgs& upd);
psgd_status check_plan(psgd_plan* plan, void* stream);
psgd_status static_workspace(psgd_plan* plan, void** ws);
// Appendix G baselines (psgd_sparse.hip): starts != nullptr: Random Block, else Random K with `indices`
psgd_status launch_sparse_step(psgd_plan* plan, const void* grad, float* err, const int64_t* starts,
                               const int64_t* indices, float* vals, void* out, void* stream);
psgd_status read_trace(psgd_plan* plan, uint64_t* out, int64_t capacity, int64_t* n_written);
psgd_status resident_check_device(psgd_plan* plan);
psgd_status launch_resident_step(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* out,
                                 void* workspace, void* stream, const UpdateArgs& upd = UpdateArgs(), int iterations = 1);
// The resident kernel's synchronisation words (units of unsigned), one 256-byte line each: an error word
// (a wait gave up), the epoch that tags this step's mailbox slots, the count of finished workgroups.
constexpr int kSyncLineWords = 64;
constexpr int64_t res_sync_err() { return 1 * kSyncLineWords; }
constexpr int64_t res_sync_epoch() { return 2 * kSyncLineWords; }
constexpr int64_t res_sync_done() { return 3 * kSyncLineWords; }
constexpr int64_t kResSyncWords = 4 * kSyncLineWords;
}  // namespace psgd

#endif
