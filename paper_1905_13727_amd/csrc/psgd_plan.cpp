// Host side of the library: plan construction (flat layout, effective ranks,
// tile work-lists, workspace layout, traffic model) and the C ABI entry points.
// No HIP call is made in this file.
#include <algorithm>
#include <cstring>
#include <new>

#include "psgd_internal.h"

namespace psgd {

static int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
static int64_t ceil_div(int64_t x, int64_t a) { return (x + a - 1) / a; }

// Split `total` items into `parts` consecutive ranges whose sizes differ by at most one.
static void even_split(int64_t total, int64_t parts, int64_t idx, int64_t* begin, int64_t* count) {
    const int64_t base = total / parts, rem = total % parts;
    *begin = idx * base + std::min(idx, rem);
    *count = base + (idx < rem ? 1 : 0);
}

// Column chunks of a row of `nvec` vectors when one wavefront lane owns at most
// `nv` vectors: chunks are whole multiples of 64 vectors except the last.
static int64_t col_chunks(int64_t nvec, int64_t nv) { return ceil_div(nvec, (int64_t)kWave * nv); }

static void col_chunk_range(int64_t nvec, int64_t nchunk, int64_t c, int32_t* vec0, int32_t* cnt) {
    const int64_t units = ceil_div(nvec, kWave);
    int64_t u0, un;
    even_split(units, nchunk, c, &u0, &un);
    const int64_t v0 = u0 * kWave;
    const int64_t v1 = std::min(nvec, (u0 + un) * kWave);
    *vec0 = (int32_t)v0;
    *cnt = (int32_t)(v1 - v0);
}

// Rows per workgroup tile of the three sweeps when the tuning leaves them to the planner (0), from sweeps on the
// three kinds of sets.  First sweep: a tile of about 8192 elements per column vector a lane owns (16 rows of
// 4-wide vectors, 32 of 2-wide, 64 of scalars).  Second sweep: 128 rows, but 1024 for matrices that are both tall
// and wide (>= 2048 each way), where fewer partial Q pay more than more workgroups.  Third sweep: 16 rows.  A small
// set (under 16 M matrix elements over all workers: each sweep lasts a few tens of microseconds) takes tiles twice
// as tall in the first and third sweep: fewer, longer-lived workgroups.
static bool small_set(const psgd_plan* plan) {
    return (int64_t)plan->workers * plan->sizes.n_mat_elems < (int64_t(16) << 20);
}
static int64_t rows_first_sweep(const psgd_plan* plan, const MatDesc& d, int64_t forced) {
    return forced > 0 ? forced : (small_set(plan) ? 2 : 1) * (64 / d.vec);
}
static int64_t rows_second_sweep(const MatDesc& d, int64_t forced) {
    return forced > 0 ? forced : (d.n >= 2048 && d.m >= 2048 ? 1024 : 128);
}
static int64_t rows_third_sweep(const psgd_plan* plan, int64_t forced) {
    return forced > 0 ? forced : (small_set(plan) ? 32 : 16);
}

// sweep: 1, 2, 3 (rows per tile by the rules above when rows_forced is 0)
static void streaming_tiles(const psgd_plan* plan, int sweep, int64_t rows_forced, int64_t nv, bool by_col_part,
                            std::vector<Tile>* out, std::vector<int32_t>* n_rblock,
                            std::vector<int32_t>* n_cchunk) {
    out->clear();
    for (size_t i = 0; i < plan->mats.size(); ++i) {
        const MatDesc& d = plan->mats[i];
        const int64_t rows_per_tile = sweep == 1 ? rows_first_sweep(plan, d, rows_forced)
                                      : (sweep == 2 ? rows_second_sweep(d, rows_forced) : rows_third_sweep(plan, rows_forced));
        const int64_t nvec = d.m / d.vec;
        const int64_t ncc = col_chunks(nvec, nv);
        const int64_t nrb = ceil_div(d.n, rows_per_tile);
        if (n_rblock) (*n_rblock)[i] = (int32_t)nrb;
        if (n_cchunk) (*n_cchunk)[i] = (int32_t)ncc;
        for (int64_t b = 0; b < nrb; ++b) {
            int64_t r0, rn;
            even_split(d.n, nrb, b, &r0, &rn);
            for (int64_t c = 0; c < ncc; ++c) {
                Tile t{};
                t.mat = (int32_t)i;
                t.row0 = (int32_t)r0;
                t.nrows = (int32_t)rn;
                col_chunk_range(nvec, ncc, c, &t.vec0, &t.nvec);
                t.part = (int32_t)(by_col_part ? c : b);
                out->push_back(t);
            }
        }
    }
}

// Workgroups are handed to the 8 accelerator dies (XCDs, one L2 each) round robin by their linear index.  With
// the tile list permuted so that entry b is the (b / 8)-th tile of the b % 8-th contiguous eighth of the list,
// each die works through one contiguous range of tiles: neighbouring tiles (column chunks of the same rows, the
// next row block) share cache lines at their edges when rows are not multiples of the line size, and those lines
// then stay within one L2 instead of being fetched and partially written back by two.
static void order_for_xcds(std::vector<Tile>& tiles) {
    constexpr size_t X = 8;
    const size_t nb = tiles.size();
    if (nb < 2 * X) return;
    const size_t per = nb / X, rem = nb % X;
    std::vector<Tile> out(nb);
    for (size_t b = 0; b < nb; ++b) {
        const size_t x = b % X, k = b / X;
        out[b] = tiles[x * per + std::min(x, rem) + k];
    }
    tiles.swap(out);
}

// The same within groups of consecutive matrices: a group is closed once it holds `min_tiles` tiles, so that a large
// matrix is spread over all dies by itself (the dies then work on the same matrix at the same time) while small
// ones are ordered together.  Slices of the vector region (mat < 0) are left where they are.
static void order_for_xcds_grouped(std::vector<Tile>& tiles, size_t min_tiles) {
    size_t b = 0;
    while (b < tiles.size()) {
        if (tiles[b].mat < 0) { ++b; continue; }
        size_t e = b;
        while (e < tiles.size() && tiles[e].mat >= 0) {
            // extend by one whole matrix
            const int32_t m = tiles[e].mat;
            while (e < tiles.size() && tiles[e].mat == m) ++e;
            if (e - b >= min_tiles) break;
        }
        std::vector<Tile> run(tiles.begin() + b, tiles.begin() + e);
        order_for_xcds(run);
        std::copy(run.begin(), run.end(), tiles.begin() + b);
        b = e;
    }
}

// xcd_order: 0 leaves a list as built, 1 orders it as a whole, k >= 2 in groups of at least k tiles.
static void order_tiles(std::vector<Tile>& tiles, int64_t xcd_order) {
    if (xcd_order >= 2) order_for_xcds_grouped(tiles, (size_t)xcd_order);
    else if (xcd_order == 1) order_for_xcds(tiles);
}

// The planner's own group size (xcd_order = -1): about 4096 workgroups per group, counting the W workers that
// every tile is launched for; between 128 and 2048 tiles.  Measured on the ResNet18-shaped set: at W = 16 groups of
// 64...256 tiles are 3-4 % faster than groups of 2048 (the sweeps' first and third kernel), at W = 4 and W = 1 the
// size makes no difference; LSTM-shaped set at W = 4: 1.5 %.
static int64_t group_tiles(const psgd_plan* plan) {
    return std::min<int64_t>(2048, std::max<int64_t>(128, 4096 / plan->workers));
}


// Matrix-core path: its own tilings and workspace layout.
static psgd_status build_hr_tables(psgd_plan* plan) {
    const Tuning& tu = plan->tuning;
    if (tu.hr_k3_rows < 64 || tu.hr_k1_rows < 64 || tu.hr_k1_rows > 256 || tu.hr_k1_rows % 64 != 0 ||
        tu.hr_k1_cols < 64 || tu.hr_k1_cols % 64 != 0 || (tu.hr_k4_rows != 0 && (tu.hr_k4_rows < 16 || tu.hr_k4_rows > 1024)) ||
        tu.stream_hints < -1 || tu.stream_hints > 1 || tu.xcd_order < -1 || tu.gram_fused < 0 || tu.gram_fused > 2 || tu.gram_spin < 1 ||
        tu.gram_spin > (1 << 24))
        return PSGD_EINVAL;
    for (const MatDesc& d : plan->mats)   // 16-byte accesses along the rows, 31-bit byte offsets within a tile
        if (d.m % 4 != 0 || d.m > kHrMaxCols || d.n > kHrMaxRows) return PSGD_EUNSUPPORTED;
    const int64_t W = plan->workers;
    const size_t nm = plan->mats.size();
    plan->tiles1.clear(); plan->tiles3.clear(); plan->tiles4.clear(); plan->tiles4u.clear(); plan->tilesp.clear();
    plan->small_mats.clear(); plan->tiles_gram.clear(); plan->tilesq.clear();
    plan->hr_tiles1.clear(); plan->hr_tiles3.clear(); plan->hr_tiles4.clear();
    plan->p_pre_reduce = false;
    const int64_t right_rows = tu.hr_k1_rows;
    // rows per workgroup of the decompression: measured best on the 24-layer transformer set at ranks 16, 32, 64
    // (one, two, four rank tiles of 16)
    // measured on the 24-layer transformer-shaped set (k_hr_decomp, ms): rank 16: 2.16 at 64 rows, 2.22 at 128, 2.25 at
    // 256; rank 32: 2.54 at 64, 2.28 at 128...256, 2.36 at 512; rank 64: 3.04 at 128, 2.62 at 256, 2.48 at 512
    const int64_t decomp_rows = tu.hr_k4_rows ? tu.hr_k4_rows : (plan->rank <= 16 ? 64 : (plan->rank <= 32 ? 256 : 512));
    int64_t pp = 0, qp = 0, gp = 0, cp = 0;
    for (size_t i = 0; i < nm; ++i) {
        MatDesc& d = plan->mats[i];
        d.n_cchunk = (int32_t)ceil_div(d.m, tu.hr_k1_cols);
        const int64_t nrb = ceil_div(d.n, tu.hr_k3_rows);
        d.n_rblock = (int32_t)nrb;   // one partial Q per row block (the workgroup adds its four strips itself)
        // Gram blocks: 128 rows each, more for very tall panels so that the one workgroup that adds up a matrix's
        // blocks has at most 64 of them
        const int64_t gram_rows = kHrGramTileRows * ceil_div(d.n, (int64_t)kHrGramTileRows * 64);
        d.n_gblock = (int32_t)ceil_div(d.n, gram_rows);
        d.ppart_off = pp;
        pp += round_up(W * d.n_cchunk * d.n * d.r, kAlignElems);
        d.gram_off = gp;
        gp += round_up((int64_t)d.n_gblock * d.r * d.r, 32);
        d.chol_off = cp;
        cp += round_up((int64_t)d.r * d.r + d.r, 32);
        for (int64_t r0 = 0; r0 < d.n; r0 += right_rows)
            for (int64_t cc = 0; cc < d.n_cchunk; ++cc) {
                Tile t{};
                t.mat = (int32_t)i; t.row0 = (int32_t)r0; t.nrows = (int32_t)std::min<int64_t>(right_rows, d.n - r0);
                t.vec0 = (int32_t)(cc * tu.hr_k1_cols);
                t.nvec = (int32_t)std::min<int64_t>(tu.hr_k1_cols, d.m - t.vec0);
                t.part = (int32_t)cc;
                plan->hr_tiles1.push_back(t);
            }
        for (int64_t b = 0; b < nrb; ++b)
            for (int64_t c0 = 0; c0 < d.m; c0 += 128) {
                Tile t{};
                t.mat = (int32_t)i; t.row0 = (int32_t)(b * tu.hr_k3_rows);
                t.nrows = (int32_t)std::min<int64_t>(tu.hr_k3_rows, d.n - t.row0);
                t.vec0 = (int32_t)c0; t.nvec = (int32_t)std::min<int64_t>(128, d.m - c0);
                t.part = (int32_t)b;
                plan->hr_tiles3.push_back(t);
            }
        for (int64_t r0 = 0; r0 < d.n; r0 += decomp_rows)
            for (int64_t c0 = 0; c0 < d.m; c0 += 128) {
                Tile t{};
                t.mat = (int32_t)i; t.row0 = (int32_t)r0; t.nrows = (int32_t)std::min<int64_t>(decomp_rows, d.n - r0);
                t.vec0 = (int32_t)c0; t.nvec = (int32_t)std::min<int64_t>(128, d.m - c0);
                plan->hr_tiles4.push_back(t);
            }
        for (int32_t b = 0; b < d.n_gblock; ++b) {
            Tile t{};
            t.mat = (int32_t)i; t.row0 = (int32_t)(b * gram_rows); t.nrows = (int32_t)std::min<int64_t>(gram_rows, d.n - t.row0);
            t.part = b;
            plan->tiles_gram.push_back(t);
        }
    }
    for (size_t i = 0; i < nm; ++i) {
        MatDesc& d = plan->mats[i];
        d.qpart_off = pp + qp;
        qp += round_up(W * d.n_rblock * d.m * d.r, kAlignElems);
        // a matrix with a single partial Q (one worker, one row block) has it written straight into Q
        const int64_t total = W * d.n_rblock > 1 ? (int64_t)d.m * d.r : 0;
        for (int64_t e = 0; e < total; e += kWave) {
            Tile t{};
            t.mat = (int32_t)i; t.elem0 = e; t.nelem = std::min<int64_t>(kWave, total - e);
            plan->tilesq.push_back(t);
        }
    }
    plan->ws_ppart_floats = pp;
    plan->ws_qpart_floats = qp;
    plan->ws_gram_doubles = gp;
    plan->ws_chol_doubles = cp;
    plan->sizes.workspace_bytes =
        std::max<int64_t>(256, round_up((pp + qp) * (int64_t)sizeof(float), 256) + (gp + cp) * (int64_t)sizeof(double));
    plan->stream_hints = tu.stream_hints < 0 ? W * plan->sizes.n_mat_elems * (int64_t)sizeof(float) > kStreamHintBytes
                                             : tu.stream_hints != 0;
    plan->resident_ok = false;
    plan->res_tiles.clear(); plan->res_mats.clear();
    plan->res_ws_floats = 0; plan->res_blocks = 0; plan->res_mail_slots = 0; plan->res_sync_words = 0;
    // Whole-list order for P = M Q and the decompression was 3 % faster than groups in one process with the buffers
    // held fixed, and no faster with the benchmark's own allocations: groups, as on the streaming path.
    const int64_t order = tu.xcd_order < 0 ? group_tiles(plan) : tu.xcd_order;
    order_tiles(plan->hr_tiles1, order);
    order_tiles(plan->hr_tiles3, order);
    order_tiles(plan->hr_tiles4, order);
    plan->tables_built = true;
    return PSGD_OK;
}

psgd_status build_tables(psgd_plan* plan) {
    const Tuning& tu = plan->tuning;
    // Ranks above 8 run on the matrix-core kernels; bf16 data at the lower ranks on either (bf16_valu).  The planner's
    // own choice for bf16 data: matrix cores at rank >= 4 on a set beyond the memory-side cache, if its shapes are ones
    // those kernels take (24-layer transformer-shaped set, ms per step, streaming / matrix cores: rank 2: 5.17 / 5.15,
    // rank 4: 5.28 / 5.17, rank 8: 6.43 / 5.19).
    const bool bf16 = plan->grad_dtype != PSGD_F32 || plan->out_dtype != PSGD_F32;
    if (tu.bf16_valu < -1 || tu.bf16_valu > 1) return PSGD_EINVAL;
    bool hr_low = bf16 && tu.bf16_valu == 0;
    if (bf16 && tu.bf16_valu < 0 && plan->rank >= 4 &&
        plan->workers * plan->sizes.n_mat_elems * (int64_t)sizeof(float) > kStreamHintBytes) {
        hr_low = true;
        for (const MatDesc& d : plan->mats)
            if (d.m % 4 != 0 || d.m > kHrMaxCols || d.n > kHrMaxRows) hr_low = false;
    }
    plan->hr = plan->rank > kValuMaxRank || hr_low;
    if (plan->hr) return build_hr_tables(plan);
    if (plan->out_dtype != PSGD_F32 && tu.k4_nv != 1) return PSGD_EINVAL;   // bf16 output: one column vector per lane
    if (tu.k1_rows < 0 || tu.k3_rows < 0 || tu.k4_rows < 0 || tu.k1_nv < 1 ||
        tu.k1_nv > kMaxVecPerLaneK1 || tu.k3_nv < 1 || tu.k3_nv > kMaxVecPerLaneK3 || tu.k4_nv < 1 ||
        tu.k4_nv > kMaxVecPerLaneK3 || tu.res_rows < 0 || tu.res_rows > kResRows || tu.resident < 0 || tu.resident > 2 ||
        tu.res_spin < 1 || tu.res_spin > (int64_t(1) << 30) || tu.res_max_blocks < 0 || tu.res_max_blocks > 65535 ||
        tu.stream_hints < -1 || tu.stream_hints > 1 || tu.xcd_order < -1 || tu.gram_fused < 0 || tu.gram_fused > 2 || tu.gram_spin < 1 ||
        tu.gram_spin > (1 << 24) || tu.ortho_rows < 0 || tu.ortho_rows > kOrthoMaxRows)
        return PSGD_EINVAL;
    const size_t nm = plan->mats.size();
    // k_ef_right and k_left address the rows of a wavefront's strip (a quarter of the tile's rows) with 31-bit
    // byte offsets
    for (const MatDesc& d : plan->mats)
        if (ceil_div(std::max(rows_first_sweep(plan, d, tu.k1_rows), rows_second_sweep(d, tu.k3_rows)), kWavesPerBlock) * d.m * 4 >=
            (int64_t(1) << 31))
            return PSGD_EUNSUPPORTED;
    std::vector<int32_t> nrb(nm, 0), ncc(nm, 0);
    streaming_tiles(plan, 1, tu.k1_rows, tu.k1_nv, true, &plan->tiles1, nullptr, &ncc);
    streaming_tiles(plan, 2, tu.k3_rows, tu.k3_nv, false, &plan->tiles3, &nrb, nullptr);
    streaming_tiles(plan, 3, tu.k4_rows, tu.k4_nv, false, &plan->tiles4, nullptr, nullptr);

    // The pass fused with the momentum / parameter update moves 20 bytes per element where the plain one moves 12 and
    // wants taller tiles on a mid-sized single-worker set (LSTM-shaped set, rank 4: 163 -> 155 us with 64 rows; the
    // ResNet18-shaped sets at 1 and 16 workers are at their optimum with the plain pass's tiles).
    plan->tiles4u.clear();
    if (tu.k4_rows == 0 && plan->workers == 1 && !small_set(plan) &&
        plan->sizes.n_mat_elems * (int64_t)sizeof(float) <= kStreamHintBytes)
        streaming_tiles(plan, 3, 64, tu.k4_nv, false, &plan->tiles4u, nullptr, nullptr);

    // vector region: slices appended to the decompress work-list
    const int64_t L = plan->sizes.n_vec_elems;
    const int64_t vec_slice = (int64_t)kBlock * 4 * 4;
    for (int64_t e = 0; e < L; e += vec_slice) {
        Tile t{};
        t.mat = -1;
        t.elem0 = e;
        t.nelem = std::min(vec_slice, L - e);
        plan->tiles4.push_back(t);
        if (!plan->tiles4u.empty()) plan->tiles4u.push_back(t);
    }

    // workspace: partial P of every matrix ([W * n_cchunk][n][r] each), then partial Q
    // ([W * n_rblock][m][r] each), then (doubles) the Gram partials of the tall panels
    const int64_t W = plan->workers;
    int64_t pp = 0, qp = 0, gp = 0;
    plan->tiles_gram.clear();
    plan->small_mats.clear();
    for (size_t i = 0; i < nm; ++i) {
        MatDesc& d = plan->mats[i];
        d.n_cchunk = ncc[i];
        d.n_rblock = nrb[i];
        d.ppart_off = pp;
        pp += round_up(W * d.n_cchunk * d.n * d.r, kAlignElems);
        if ((int64_t)d.n * d.r <= kPanelFloats && d.n <= tu.ortho_rows) {
            d.n_gblock = 0;
            d.gram_off = 0;
            plan->small_mats.push_back((int32_t)i);
        } else {
            d.n_gblock = (int32_t)ceil_div(d.n, kGramRows);
            d.gram_off = gp;
            gp += round_up((int64_t)d.n_gblock * d.r * d.r, 32);
            for (int32_t b = 0; b < d.n_gblock; ++b) {
                Tile t{};
                t.mat = (int32_t)i;
                t.row0 = b * kGramRows;
                t.nrows = std::min<int32_t>(kGramRows, d.n - t.row0);
                t.part = b;
                plan->tiles_gram.push_back(t);
            }
        }
    }
    for (size_t i = 0; i < nm; ++i) {
        MatDesc& d = plan->mats[i];
        d.qpart_off = pp + qp;
        qp += round_up(W * d.n_rblock * d.m * d.r, kAlignElems);
    }
    plan->ws_ppart_floats = pp;
    plan->ws_qpart_floats = qp;
    plan->ws_gram_doubles = gp;
    plan->sizes.workspace_bytes =
        std::max<int64_t>(256, round_up((pp + qp) * (int64_t)sizeof(float), 256) + gp * (int64_t)sizeof(double));

    // the same slicing of the n x r panels, used when a matrix has many partial-P slices
    plan->tilesp.clear();
    plan->p_pre_reduce = false;
    for (size_t i = 0; i < nm; ++i) {
        const MatDesc& d = plan->mats[i];
        if (W * d.n_cchunk > kPreReduceParts) plan->p_pre_reduce = true;
        const int64_t total = (int64_t)d.n * d.r;
        for (int64_t e = 0; e < total; e += kWave) {
            Tile t{};
            t.mat = (int32_t)i;
            t.elem0 = e;
            t.nelem = std::min<int64_t>(kWave, total - e);
            plan->tilesp.push_back(t);
        }
    }
    // Q reduction: slices of 64 elements of each matrix's m x r panel (4 part-slices per element in a workgroup)
    plan->tilesq.clear();
    for (size_t i = 0; i < nm; ++i) {
        const MatDesc& d = plan->mats[i];
        const int64_t total = (int64_t)d.m * d.r;
        for (int64_t e = 0; e < total; e += kWave) {
            Tile t{};
            t.mat = (int32_t)i;
            t.elem0 = e;
            t.nelem = std::min<int64_t>(kWave, total - e);
            plan->tilesq.push_back(t);
        }
    }
    plan->stream_hints = tu.stream_hints < 0 ? W * plan->sizes.n_mat_elems * (int64_t)sizeof(float) > kStreamHintBytes
                                             : tu.stream_hints != 0;
    build_resident(plan, (int64_t)kResCUs * kResBlocksPerCU);
    plan->sizes.workspace_bytes =
        std::max<int64_t>(plan->sizes.workspace_bytes, plan->res_ws_floats * (int64_t)sizeof(float));
    // The planner's own choice: groups; for one worker and a set beyond the memory-side cache the whole list instead
    // (24-layer transformer set, rank 4: k_left 880 -> 842 us, k_decomp 2186 -> 2143 us, k_ef_right 2203 -> 2217 us,
    // the step 5.34 -> 5.28 ms; with the first sweep alone left in groups the second sweep's gain is lost; at 16
    // workers whole-list order loses 1-3 % in every sweep).
    const int64_t order = tu.xcd_order >= 0 ? tu.xcd_order : (W == 1 && plan->stream_hints ? 1 : group_tiles(plan));
    order_tiles(plan->tiles1, order);
    order_tiles(plan->tiles3, order);
    order_tiles(plan->tiles4, order);
    order_tiles(plan->tiles4u, order);
    plan->tables_built = true;
    return PSGD_OK;
}

// Resident tiling: every matrix is cut into strips of at most `h` rows and chunks of 64 column
// vectors; one wavefront keeps one (strip, chunk) tile in registers for the whole step.  The model
// qualifies when all tiles fit the wavefront slots of one co-resident grid.
static int64_t resident_tiles_for(const psgd_plan* plan, int h) {
    int64_t total = 0;
    for (const MatDesc& d : plan->mats) total += ceil_div(d.n, h) * ceil_div(d.m / d.vec, kWave);
    return total;
}

void build_resident(psgd_plan* plan, int64_t device_blocks) {
    plan->resident_ok = false;
    plan->res_tiles.clear();
    plan->res_mats.clear();
    plan->res_ws_floats = 0;
    plan->res_blocks = 0;
    const Tuning& tu = plan->tuning;
    if (!tu.resident || plan->workers != 1 || plan->rank > kResMaxRank || plan->mats.empty()) return;
    if (plan->grad_dtype != PSGD_F32 || plan->out_dtype != PSGD_F32) return;
    for (const MatDesc& d : plan->mats)
        if (d.n > kResMaxN) return;
    const int64_t max_blocks = tu.res_max_blocks > 0 ? tu.res_max_blocks : device_blocks;
    const int64_t L = plan->sizes.n_vec_elems;
    const int64_t vec_slice = (int64_t)kWave * 4 * 8;   // elements of the vector region per wavefront
    const int64_t vec_tiles = ceil_div(L, vec_slice);

    // The matrices keep model order in the tile list (largest first, so that the matrices with the most strips and
    // column chunks sit in the first workgroups, was 1 % slower on the ResNet18-shaped set).
    auto layout = [&](int h, std::vector<RTile>* tiles, std::vector<MatDesc>* mats, int32_t* n_cntq,
                      int32_t* n_cnts) -> int64_t {
        // returns the number of workgroups, fills the tables when tiles != nullptr
        int64_t slots = 0;            // wavefront slots used so far (multiple of 4 at block boundaries)
        int32_t cntq = 0, cnts = 0;
        int cur_vec = 0;
        if (mats) mats->assign(plan->mats.size(), MatDesc{});
        auto pad_block = [&]() {
            while (slots % kWavesPerBlock) {
                if (tiles) { RTile t{}; t.mat = -2; tiles->push_back(t); }
                ++slots;
            }
        };
        for (size_t i = 0; i < plan->mats.size(); ++i) {
            const MatDesc& d0 = plan->mats[i];
            if (d0.vec != cur_vec) { pad_block(); cur_vec = d0.vec; }
            const int64_t nvec = d0.m / d0.vec;
            const int64_t nchunk = ceil_div(nvec, kWave);
            const int64_t nstrip = ceil_div(d0.n, h);
            int32_t max_runs = 0;
            const size_t first_tile = tiles ? tiles->size() : 0;
            for (int64_t c = 0; c < nchunk; ++c) {
                int32_t runs = 0;
                size_t run_leader = 0;
                const size_t chunk_first = tiles ? tiles->size() : 0;
                for (int64_t sidx = 0; sidx < nstrip; ++sidx) {
                    int64_t r0, rn;
                    even_split(d0.n, nstrip, sidx, &r0, &rn);
                    const bool new_run = (sidx == 0) || (slots % kWavesPerBlock == 0);
                    if (tiles) {
                        RTile t{};
                        t.mat = (int32_t)i;
                        t.row0 = (int32_t)r0;
                        t.nrows = (int32_t)rn;
                        t.vec0 = (int32_t)(c * kWave);
                        t.nvec = (int32_t)std::min<int64_t>(kWave, nvec - c * kWave);
                        t.ppart = (int32_t)c;
                        t.cntq = cntq;
                        t.cnts = cnts + (int32_t)sidx;
                        if (new_run) {
                            run_leader = tiles->size();
                            t.qrun_len = 1;
                            t.qpart = runs;
                        } else {
                            (*tiles)[run_leader].qrun_len += 1;
                        }
                        tiles->push_back(t);
                    }
                    if (new_run) ++runs;
                    ++slots;
                }
                if (tiles)
                    for (size_t k = chunk_first; k < tiles->size(); ++k) (*tiles)[k].nqparts = runs;
                max_runs = std::max(max_runs, runs);
                ++cntq;
            }
            if (tiles) {
                for (size_t k = first_tile; k < tiles->size(); ++k)
                    if ((*tiles)[k].mat == (int32_t)i) (*tiles)[k].nstrips_mat = (int32_t)nstrip;
                MatDesc d = d0;
                d.n_cchunk = (int32_t)nchunk;
                d.n_rblock = max_runs;
                (*mats)[i] = d;
            }
            cnts += (int32_t)nstrip;
        }
        if (vec_tiles) {
            pad_block();
            for (int64_t v = 0; v < vec_tiles; ++v) {
                if (tiles) {
                    RTile t{};
                    t.mat = -1;
                    t.elem0 = v * vec_slice;
                    t.nelem = std::min(vec_slice, L - v * vec_slice);
                    tiles->push_back(t);
                }
                ++slots;
            }
        }
        pad_block();
        if (n_cntq) *n_cntq = cntq;
        if (n_cnts) *n_cnts = cnts;
        return slots / kWavesPerBlock;
    };

    int h = 0;
    const int max_rows = res_rows_for_rank(plan->rank);
    if (tu.res_rows > 0) {
        if (tu.res_rows > max_rows) return;
        h = (int)tu.res_rows;
        if (layout(h, nullptr, nullptr, nullptr, nullptr) > max_blocks) return;
    } else {
        for (int cand = kResMinRows; cand <= max_rows; ++cand) {
            if (layout(cand, nullptr, nullptr, nullptr, nullptr) <= max_blocks) { h = cand; break; }
        }
        if (!h) return;
    }
    int32_t n_cntq = 0, n_cnts = 0;
    const int64_t blocks = layout(h, &plan->res_tiles, &plan->res_mats, &n_cntq, &n_cnts);
    plan->res_strip_rows = h;
    plan->res_blocks = (int32_t)blocks;
    plan->res_n_cntq = n_cntq;
    plan->res_n_cnts = n_cnts;
    // mailbox of the resident kernel (64-bit slots): per matrix [partial P | mean P | P_hat], then per
    // matrix [partial Q | Q]; the offsets are kept in res_mats
    int64_t off = 0;
    for (MatDesc& d : plan->res_mats) {
        d.ppart_off = off;
        off += round_up(((int64_t)d.n_cchunk + 2) * d.n * d.r, kAlignElems);
    }
    for (MatDesc& d : plan->res_mats) {
        d.qpart_off = off;
        off += round_up(((int64_t)d.n_rblock + 1) * d.m * d.r, kAlignElems);
    }
    plan->res_mail_slots = off;
    plan->res_ws_floats = 0;   // nothing of the caller's workspace is used
    plan->res_sync_words = kResSyncWords;
    plan->resident_ok = true;
}

}  // namespace psgd

using namespace psgd;

extern "C" {

psgd_status psgd_plan_create(const psgd_shape* shapes, int32_t n_tensors, int32_t rank, int32_t workers,
                             psgd_dtype grad_dtype, psgd_dtype out_dtype, psgd_plan** out_plan) {
    if (!out_plan) return PSGD_EINVAL;
    *out_plan = nullptr;
    if (!shapes || n_tensors < 1 || rank < 1 || workers < 1) return PSGD_EINVAL;
    if ((grad_dtype != PSGD_F32 && grad_dtype != PSGD_BF16) ||
        (out_dtype != PSGD_F32 && out_dtype != PSGD_BF16))
        return PSGD_EINVAL;
    for (int32_t t = 0; t < n_tensors; ++t) {
        if (shapes[t].rows < 1 || shapes[t].cols < 1) return PSGD_EINVAL;
        if (shapes[t].rows > INT32_MAX || shapes[t].cols > INT32_MAX) return PSGD_EUNSUPPORTED;
    }
    if (rank > PSGD_MAX_RANK) return PSGD_EUNSUPPORTED;
    // the matrix-core kernels (ranks above 8) need row lengths that are multiples of 4 and short enough for 32-bit
    // byte offsets within a tile of rows
    const bool needs_hr = rank > kValuMaxRank;
    if (needs_hr)
        for (int32_t t = 0; t < n_tensors; ++t)
            if (shapes[t].cols != 1 && (shapes[t].cols % 4 != 0 || shapes[t].cols > kHrMaxCols ||
                                        shapes[t].rows > kHrMaxRows))
                return PSGD_EUNSUPPORTED;

    psgd_plan* plan = new (std::nothrow) psgd_plan();
    if (!plan) return PSGD_ENOMEM;
    try {
        plan->rank = rank;
        plan->workers = workers;
        plan->hr = rank > kValuMaxRank;   // settled in build_tables
        plan->hr_nt = rank <= 16 ? 1 : (rank <= 32 ? 2 : 4);
        plan->grad_dtype = grad_dtype;
        plan->out_dtype = out_dtype;
        plan->shapes.assign(shapes, shapes + n_tensors);
        plan->tensor_flat_off.assign(n_tensors, 0);
        plan->tensor_mat.assign(n_tensors, -1);

        const int64_t gsz = grad_dtype == PSGD_BF16 ? 2 : 4;
        const int64_t osz = out_dtype == PSGD_BF16 ? 2 : 4;
        int64_t N = 0, P = 0, Q = 0, payload = 0, compressed = 0, kept_total = 0;
        // matrices first
        for (int32_t t = 0; t < n_tensors; ++t) {
            if (shapes[t].cols == 1) continue;
            MatDesc d{};
            d.n = (int32_t)shapes[t].rows;
            d.m = (int32_t)shapes[t].cols;
            d.r = std::min<int32_t>(rank, std::min(d.n, d.m));
            d.vec = (d.m % 4 == 0) ? 4 : (d.m % 2 == 0 ? 2 : 1);
            d.off = N;
            d.p_off = P;
            d.q_off = Q;
            d.tensor = t;
            plan->tensor_flat_off[t] = N;
            const int32_t mi = (int32_t)plan->mats.size();
            plan->tensor_mat[t] = mi;
            plan->max_n = std::max(plan->max_n, d.n);
            const int64_t elems = (int64_t)d.n * d.m;
            // Appendix G baselines: b = (n + m) r entries per matrix "to match rank-r PowerSGD", at most all of them
            d.kept = std::min(((int64_t)d.n + d.m) * rank, elems);
            d.kept_off = kept_total;
            kept_total += d.kept;
            plan->mats.push_back(d);
            for (int64_t j0 = 0; j0 < d.kept; j0 += kBlock) {
                plan->kept_slice_mat.push_back(mi);
                plan->kept_slice_first.push_back(j0);
            }
            plan->mat_tensor.push_back(t);
            // slices of the flattened matrix for their elementwise sweep: only their running count is kept (the
            // kernel finds its matrix by bisection), not a table of a million entries for a large model
            plan->flat_first.push_back(plan->flat_tiles);
            plan->flat_tiles += ceil_div(elems, kFlatTileElems);
            N += round_up(elems, kAlignElems);
            P += round_up((int64_t)d.n * d.r, kFactorAlignElems);   // every factor starts 16-byte aligned
            Q += round_up((int64_t)d.m * d.r, kFactorAlignElems);
            payload += elems;
            compressed += (int64_t)d.r * ((int64_t)d.n + d.m);
        }
        int64_t L = 0;
        int64_t nvec_t = 0;
        for (int32_t t = 0; t < n_tensors; ++t) {
            if (shapes[t].cols != 1) continue;
            plan->tensor_flat_off[t] = N + L;
            L += shapes[t].rows;
            ++nvec_t;
        }
        plan->flat_first.push_back(plan->flat_tiles);   // one past the last matrix: where the vector region's slices start
        plan->flat_vec_tiles = ceil_div(L, kFlatTileElems);
        psgd_sizes& s = plan->sizes;
        s.kept_elems = kept_total;
        plan->kept_slices = (int64_t)plan->kept_slice_mat.size();
        s.n_mat_elems = N;
        s.n_vec_elems = L;
        s.grad_stride = round_up(N + L, kAlignElems);
        s.err_stride = N;
        s.out_elems = N + L;
        s.p_elems = P;
        s.q_elems = Q;
        s.n_matrices = (int64_t)plan->mats.size();
        s.n_vectors = nvec_t;
        s.payload_elems = payload + L;
        s.compressed_elems = compressed + L;
        const int64_t W = workers;
        s.bytes_min = payload * (W * (gsz + 4 + 4) + osz) + L * (W * gsz + osz);
        s.bytes_stream = s.bytes_min + payload * W * 12;
        psgd_status st = build_tables(plan);
        if (st != PSGD_OK) {
            delete plan;
            return st;
        }
    } catch (const std::bad_alloc&) {
        delete plan;
        return PSGD_ENOMEM;
    }
    *out_plan = plan;
    return PSGD_OK;
}

void psgd_plan_destroy(psgd_plan* plan) {
    if (!plan) return;
    free_tables(plan);
    delete plan;
}

psgd_status psgd_plan_sizes(const psgd_plan* plan, psgd_sizes* out_sizes) {
    if (!plan || !out_sizes) return PSGD_EINVAL;
    *out_sizes = plan->sizes;
    return PSGD_OK;
}

psgd_status psgd_plan_offsets(const psgd_plan* plan, int32_t tensor, int64_t* flat_off, int64_t* p_off,
                              int64_t* q_off, int32_t* eff_rank) {
    if (!plan || tensor < 0 || tensor >= (int32_t)plan->shapes.size()) return PSGD_EINVAL;
    if (flat_off) *flat_off = plan->tensor_flat_off[tensor];
    const int32_t mi = plan->tensor_mat[tensor];
    if (mi < 0) {
        if (p_off) *p_off = -1;
        if (q_off) *q_off = -1;
        if (eff_rank) *eff_rank = 0;
    } else {
        const MatDesc& d = plan->mats[mi];
        if (p_off) *p_off = d.p_off;
        if (q_off) *q_off = d.q_off;
        if (eff_rank) *eff_rank = d.r;
    }
    return PSGD_OK;
}

psgd_status psgd_plan_kept(const psgd_plan* plan, int32_t tensor, int64_t* kept_off, int64_t* kept) {
    if (!plan || tensor < 0 || tensor >= (int32_t)plan->shapes.size()) return PSGD_EINVAL;
    const int32_t mi = plan->tensor_mat[tensor];
    if (kept_off) *kept_off = mi < 0 ? -1 : plan->mats[mi].kept_off;
    if (kept) *kept = mi < 0 ? 0 : plan->mats[mi].kept;
    return PSGD_OK;
}

psgd_status psgd_plan_path(const psgd_plan* plan, int32_t* path) {
    if (!plan || !path) return PSGD_EINVAL;
    *path = plan->hr ? PSGD_PATH_MATRIX_CORES : (plan->resident_ok ? PSGD_PATH_RESIDENT : PSGD_PATH_STREAMING);
    return PSGD_OK;
}

psgd_status psgd_random_block_step(psgd_plan* plan, const void* grad, float* err, const int64_t* starts, float* vals,
                                   void* out, void* hip_stream) {
    if (!plan || !grad || !err || !starts || !vals || !out) return PSGD_EINVAL;
    if (plan->grad_dtype != PSGD_F32 || plan->out_dtype != PSGD_F32) return PSGD_EUNSUPPORTED;
    return launch_sparse_step(plan, grad, err, starts, nullptr, vals, out, hip_stream);
}

psgd_status psgd_random_k_step(psgd_plan* plan, const void* grad, float* err, const int64_t* indices, float* vals,
                               void* out, void* hip_stream) {
    if (!plan || !grad || !err || !indices || !vals || !out) return PSGD_EINVAL;
    if (plan->grad_dtype != PSGD_F32 || plan->out_dtype != PSGD_F32) return PSGD_EUNSUPPORTED;
    return launch_sparse_step(plan, grad, err, nullptr, indices, vals, out, hip_stream);
}

psgd_status psgd_plan_set_tuning(psgd_plan* plan, const char* key, int64_t value) {
    if (!plan || !key) return PSGD_EINVAL;
    if (plan->uploaded) return PSGD_EINVAL;
    Tuning tu = plan->tuning;
    if (!strcmp(key, "k1_rows")) tu.k1_rows = value;
    else if (!strcmp(key, "k1_nv")) tu.k1_nv = value;
    else if (!strcmp(key, "k3_rows")) tu.k3_rows = value;
    else if (!strcmp(key, "k3_nv")) tu.k3_nv = value;
    else if (!strcmp(key, "k4_rows")) tu.k4_rows = value;
    else if (!strcmp(key, "k4_nv")) tu.k4_nv = value;
    else if (!strcmp(key, "hr_k3_rows")) tu.hr_k3_rows = value;
    else if (!strcmp(key, "xcd_order")) tu.xcd_order = value;
    else if (!strcmp(key, "hr_k4_rows")) tu.hr_k4_rows = value;
    else if (!strcmp(key, "hr_k1_rows")) tu.hr_k1_rows = value;
    else if (!strcmp(key, "hr_k1_cols")) tu.hr_k1_cols = value;
    else if (!strcmp(key, "resident")) tu.resident = value;
    else if (!strcmp(key, "stream_hints")) tu.stream_hints = value;
    else if (!strcmp(key, "bf16_valu")) tu.bf16_valu = value;
    else if (!strcmp(key, "gram_fused")) tu.gram_fused = value;
    else if (!strcmp(key, "gram_spin")) tu.gram_spin = value;
    else if (!strcmp(key, "ortho_rows")) tu.ortho_rows = value;
    else if (!strcmp(key, "res_rows")) tu.res_rows = value;
    else if (!strcmp(key, "res_trace")) tu.res_trace = value;
    else if (!strcmp(key, "res_spin")) tu.res_spin = value;
    else if (!strcmp(key, "res_max_blocks")) tu.res_max_blocks = value;
    else return PSGD_EINVAL;
    Tuning old = plan->tuning;
    plan->tuning = tu;
    try {
        psgd_status st = build_tables(plan);
        if (st != PSGD_OK) {
            plan->tuning = old;
            build_tables(plan);
        }
        return st;
    } catch (const std::bad_alloc&) {
        return PSGD_ENOMEM;
    }
}

static bool bad_ptrs(const void* a, const void* b, const void* c, const void* d, const void* e) {
    return !a || !b || !c || !d || !e;
}

psgd_status psgd_compress(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* workspace,
                          void* hip_stream) {
    if (!plan || bad_ptrs(grad, err, q, p, workspace)) return PSGD_EINVAL;
    return launch_compress(plan, grad, err, q, p, workspace, hip_stream);
}

psgd_status psgd_decompress(psgd_plan* plan, const float* p, const float* q, float* err, const void* grad,
                            void* out, void* workspace, void* hip_stream) {
    if (!plan || bad_ptrs(p, q, err, out, workspace) || !grad) return PSGD_EINVAL;
    return launch_decompress(plan, p, q, err, grad, out, workspace, hip_stream);
}

psgd_status psgd_step(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* out,
                      void* workspace, void* hip_stream) {
    if (!plan || bad_ptrs(grad, err, q, p, workspace) || !out) return PSGD_EINVAL;
    if (plan->resident_ok) return launch_resident_step(plan, grad, err, q, p, out, workspace, hip_stream);
    psgd_status st = launch_compress(plan, grad, err, q, p, workspace, hip_stream);
    if (st != PSGD_OK) return st;
    return launch_decompress(plan, p, q, err, grad, out, workspace, hip_stream);
}

psgd_status psgd_step_static(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* out,
                             void* hip_stream) {
    if (!plan || !grad || !err || !q || !p || !out) return PSGD_EINVAL;
    void* ws = nullptr;
    psgd_status st = static_workspace(plan, &ws);
    if (st != PSGD_OK) return st;
    return psgd_step(plan, grad, err, q, p, out, ws, hip_stream);
}

psgd_status psgd_step_iterations(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* out,
                                 void* workspace, void* hip_stream, int32_t iterations) {
    if (!plan || bad_ptrs(grad, err, q, p, workspace) || !out || iterations < 1 || iterations > 64) return PSGD_EINVAL;
    if (plan->resident_ok) return launch_resident_step(plan, grad, err, q, p, out, workspace, hip_stream, UpdateArgs(), iterations);
    psgd_status st = launch_compress(plan, grad, err, q, p, workspace, hip_stream);
    for (int32_t it = 1; it < iterations && st == PSGD_OK; ++it)
        st = launch_compress(plan, err, err, q, p, workspace, hip_stream, false);
    if (st != PSGD_OK) return st;
    return launch_decompress(plan, p, q, err, grad, out, workspace, hip_stream);
}

psgd_status psgd_iterate(psgd_plan* plan, float* err, float* q, float* p, void* workspace, void* hip_stream) {
    if (!plan || !err || !q || !p || !workspace) return PSGD_EINVAL;
    // the gradient pointer is not dereferenced when nothing is added; err stands in so that it is never null
    return launch_compress(plan, err, err, q, p, workspace, hip_stream, false);
}

static bool update_args(const psgd_plan* plan, float* mom, float* param, float lr, float momentum, UpdateArgs* upd) {
    (void)plan;
    if (!mom || !param || !(lr == lr) || !(momentum == momentum)) return false;   // null or NaN
    upd->mom = mom;
    upd->param = param;
    upd->lr = lr;
    upd->lam = momentum;
    return true;
}

psgd_status psgd_decompress_update(psgd_plan* plan, const float* p, const float* q, float* err, const void* grad,
                                   float* mom, float* param, float lr, float momentum, void* workspace,
                                   void* hip_stream) {
    UpdateArgs upd;
    if (!plan || !p || !q || !err || !grad || !workspace || !update_args(plan, mom, param, lr, momentum, &upd))
        return PSGD_EINVAL;
    return launch_decompress(plan, p, q, err, grad, nullptr, workspace, hip_stream, upd);
}

psgd_status psgd_step_update(psgd_plan* plan, const void* grad, float* err, float* q, float* p, float* mom,
                             float* param, float lr, float momentum, void* workspace, void* hip_stream) {
    UpdateArgs upd;
    if (!plan || bad_ptrs(grad, err, q, p, workspace) || !update_args(plan, mom, param, lr, momentum, &upd))
        return PSGD_EINVAL;
    if (plan->resident_ok) return launch_resident_step(plan, grad, err, q, p, nullptr, workspace, hip_stream, upd);
    psgd_status st = launch_compress(plan, grad, err, q, p, workspace, hip_stream);
    if (st != PSGD_OK) return st;
    return launch_decompress(plan, p, q, err, grad, nullptr, workspace, hip_stream, upd);
}

psgd_status psgd_plan_set_profiling(psgd_plan* plan, int32_t enable) {
    if (!plan) return PSGD_EINVAL;
    return set_profiling(plan, enable != 0);
}

psgd_status psgd_plan_kernel_times(psgd_plan* plan, double* ms_sum, int64_t* steps) {
    if (!plan || !ms_sum || !steps) return PSGD_EINVAL;
    for (int i = 0; i < PSGD_N_KERNELS; ++i) {
        ms_sum[i] = plan->kernel_ms[i];
        plan->kernel_ms[i] = 0.0;
    }
    *steps = plan->profiled_steps;
    plan->profiled_steps = 0;
    return PSGD_OK;
}

const char* psgd_kernel_name(int32_t index) {
    static const char* const names[PSGD_N_KERNELS] = {"k_ef_right", "k_ortho",    "k_left",        "k_q_reduce",
                                                      "k_decomp",   "k_resident", "k_ef_add_zero", "k_kept_entries"};
    return (index >= 0 && index < PSGD_N_KERNELS) ? names[index] : nullptr;
}

psgd_status psgd_plan_check(psgd_plan* plan, void* hip_stream, int32_t* is_resident) {
    if (!plan) return PSGD_EINVAL;
    if (is_resident) *is_resident = plan->resident_ok ? 1 : 0;
    return check_plan(plan, hip_stream);
}

psgd_status psgd_plan_read_trace(psgd_plan* plan, uint64_t* out, int64_t capacity, int64_t* n_written) {
    if (!plan || !out || !n_written || capacity < 0) return PSGD_EINVAL;
    return read_trace(plan, out, capacity, n_written);
}

const char* psgd_status_string(psgd_status status) {
    switch (status) {
        case PSGD_OK: return "ok";
        case PSGD_EINVAL: return "invalid argument";
        case PSGD_ENOMEM: return "out of memory";
        case PSGD_EHIP: return "HIP runtime error";
        case PSGD_EUNSUPPORTED: return "unsupported";
    }
    return "unknown status";
}

const char* psgd_plan_last_error(const psgd_plan* plan) { return plan ? plan->last_error.c_str() : ""; }

}  // extern "C"
