// Host-only check of the planner's work-lists, built with g++ and the sanitizers by
// tests/test_host_planner.py.  For a set of shape lists and tunings it verifies that the
// tiles of every streaming kernel cover every matrix element exactly once, stay inside the
// row, respect the per-lane vector limit, and that every partial-sum slice lies inside the
// workspace the plan asks for: the bounds the kernels rely on.
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <utility>
#include <vector>

#include "psgd_internal.h"

namespace psgd {
void free_tables(psgd_plan*) {}
psgd_status set_profiling(psgd_plan*, bool) { return PSGD_EHIP; }
psgd_status check_plan(psgd_plan*, void*) { return PSGD_EHIP; }
psgd_status launch_sparse_step(psgd_plan*, const void*, float*, const int64_t*, const int64_t*, float*, void*, void*) {
    return PSGD_EHIP;
}
psgd_status static_workspace(psgd_plan*, void**) { return PSGD_EHIP; }
psgd_status read_trace(psgd_plan*, uint64_t*, int64_t, int64_t*) { return PSGD_EHIP; }
psgd_status launch_resident_step(psgd_plan*, const void*, float*, float*, float*, void*, void*, void*, const UpdateArgs&, int) {
    return PSGD_EHIP;
}
psgd_status launch_compress(psgd_plan*, const void*, float*, float*, float*, void*, void*, bool) { return PSGD_EHIP; }
psgd_status launch_decompress(psgd_plan*, const float*, const float*, float*, const void*, void*, void*, void*,
                              const UpdateArgs&) {
    return PSGD_EHIP;
}
}  // namespace psgd

#define CHECK(c)                                                        \
    do {                                                                \
        if (!(c)) {                                                     \
            std::printf("FAIL %s:%d %s\n", __FILE__, __LINE__, #c);     \
            std::exit(1);                                               \
        }                                                               \
    } while (0)

using namespace psgd;

// parts: 1 = column-chunk partials (P = M Q), 2 = row-block partials (Q = M^T P), 0 = the kernel writes no partials
static void check_cover(const psgd_plan* plan, const std::vector<Tile>& tiles, int nv_cap, int parts) {
    std::vector<std::vector<unsigned char>> seen(plan->mats.size());
    for (size_t i = 0; i < plan->mats.size(); ++i) seen[i].assign((size_t)plan->mats[i].n * plan->mats[i].m, 0);
    int64_t vec_seen = 0;
    std::vector<unsigned char> vseen((size_t)plan->sizes.n_vec_elems, 0);
    for (const Tile& t : tiles) {
        if (t.mat < 0) {   // a slice of the vector-shaped tensors; the list may be in any order (it is ordered for the dies)
            CHECK(t.elem0 >= 0 && t.nelem > 0 && t.elem0 + t.nelem <= plan->sizes.n_vec_elems);
            for (int64_t e = t.elem0; e < t.elem0 + t.nelem; ++e) {
                CHECK(vseen[(size_t)e] == 0);
                vseen[(size_t)e] = 1;
            }
            vec_seen += t.nelem;
            continue;
        }
        CHECK(t.mat < (int)plan->mats.size());
        const MatDesc& d = plan->mats[t.mat];
        CHECK(d.m % d.vec == 0);
        CHECK(t.nrows > 0 && t.row0 >= 0 && t.row0 + t.nrows <= d.n);
        CHECK(t.nvec > 0 && t.vec0 >= 0 && (int64_t)(t.vec0 + t.nvec) * d.vec <= d.m);
        CHECK(t.nvec <= kWave * nv_cap);
        if (parts) CHECK(t.part >= 0 && t.part < (parts == 1 ? d.n_cchunk : d.n_rblock));
        for (int i = t.row0; i < t.row0 + t.nrows; ++i)
            for (int j = t.vec0 * d.vec; j < (t.vec0 + t.nvec) * d.vec; ++j) {
                unsigned char& s = seen[t.mat][(size_t)i * d.m + j];
                CHECK(s == 0);
                s = 1;
            }
    }
    for (auto& v : seen)
        for (unsigned char s : v) CHECK(s == 1);
    if (vec_seen) CHECK(vec_seen == plan->sizes.n_vec_elems);
}

// Resident tiling: what the resident kernel relies on.
static void check_resident(const psgd_plan* plan) {
    if (!plan->resident_ok) return;
    CHECK(plan->workers == 1 && plan->rank <= kResMaxRank);
    CHECK(plan->res_blocks > 0 && plan->res_blocks <= kResCUs * kResBlocksPerCU);
    CHECK((int64_t)plan->res_tiles.size() == (int64_t)plan->res_blocks * kWavesPerBlock);
    CHECK(plan->res_mats.size() == plan->mats.size());
    std::vector<std::vector<unsigned char>> seen(plan->mats.size());
    std::vector<int> tiles_of(plan->mats.size(), 0);
    for (size_t i = 0; i < plan->mats.size(); ++i) seen[i].assign((size_t)plan->mats[i].n * plan->mats[i].m, 0);
    std::vector<int> q_leaders(plan->res_n_cntq, 0), q_expect(plan->res_n_cntq, -1);
    int64_t vec_seen = 0;
    for (int b = 0; b < plan->res_blocks; ++b) {
        const RTile* blk = &plan->res_tiles[(size_t)b * kWavesPerBlock];
        CHECK(blk[0].mat != -2);   // the first slot of a workgroup is never idle
        int vec = 0;
        for (int w = 0; w < kWavesPerBlock; ++w) {
            const RTile& t = blk[w];
            if (t.mat == -2) { CHECK(t.qrun_len == 0); continue; }
            if (t.mat == -1) {
                CHECK(t.elem0 == vec_seen && t.nelem > 0 && t.qrun_len == 0);
                vec_seen += t.nelem;
                continue;
            }
            CHECK(t.mat >= 0 && t.mat < (int)plan->mats.size());
            const MatDesc& d = plan->res_mats[t.mat];
            CHECK(d.n <= kResMaxN);
            if (!vec) vec = d.vec;
            CHECK(vec == d.vec);   // one access width per workgroup
            CHECK(t.nrows > 0 && t.nrows <= res_rows_for_rank(plan->rank) && t.row0 >= 0 && t.row0 + t.nrows <= d.n);
            CHECK(t.nvec > 0 && t.nvec <= kWave && t.vec0 >= 0 && (int64_t)(t.vec0 + t.nvec) * d.vec <= d.m);
            CHECK(t.ppart >= 0 && t.ppart < d.n_cchunk);
            CHECK(t.cntq >= 0 && t.cntq < plan->res_n_cntq);
            CHECK(t.nqparts >= 1 && t.nqparts <= d.n_rblock);
            if (q_expect[t.cntq] < 0) q_expect[t.cntq] = t.nqparts;
            CHECK(q_expect[t.cntq] == t.nqparts);
            if (t.qrun_len > 0) {
                CHECK(w + t.qrun_len <= kWavesPerBlock);
                CHECK(t.qpart >= 0 && t.qpart < t.nqparts);
                for (int k = 1; k < t.qrun_len; ++k) {
                    const RTile& f = blk[w + k];   // followers: same matrix, same column chunk, no run of their own
                    CHECK(f.mat == t.mat && f.vec0 == t.vec0 && f.nvec == t.nvec && f.qrun_len == 0 && f.cntq == t.cntq);
                }
                q_leaders[t.cntq] += 1;
            } else {
                CHECK(w > 0);
            }
            tiles_of[t.mat] += 1;
            for (int i = t.row0; i < t.row0 + t.nrows; ++i)
                for (int j = t.vec0 * d.vec; j < (t.vec0 + t.nvec) * d.vec; ++j) {
                    unsigned char& sflag = seen[t.mat][(size_t)i * d.m + j];
                    CHECK(sflag == 0);
                    sflag = 1;
                }
        }
    }
    for (auto& v : seen)
        for (unsigned char sflag : v) CHECK(sflag == 1);
    CHECK(vec_seen == plan->sizes.n_vec_elems);
    for (int c = 0; c < plan->res_n_cntq; ++c) CHECK(q_leaders[c] == q_expect[c]);   // every slot is written once
    for (const RTile& t : plan->res_tiles)
        if (t.mat >= 0) {
            const MatDesc& d = plan->res_mats[t.mat];
            CHECK(t.nstrips_mat * d.n_cchunk == tiles_of[t.mat]);
            CHECK(t.cnts >= 0 && t.cnts < plan->res_n_cnts);
            CHECK(t.nrows * d.r <= 2 * kWave);
        }
    {
        // mailbox regions: [partial P | mean P | P_hat] and [partial Q | Q] per matrix, disjoint, inside the mailbox
        std::vector<std::pair<int64_t, int64_t>> regions;
        for (const MatDesc& d : plan->res_mats) {
            regions.push_back({d.ppart_off, d.ppart_off + ((int64_t)d.n_cchunk + 2) * d.n * d.r});
            regions.push_back({d.qpart_off, d.qpart_off + ((int64_t)d.n_rblock + 1) * d.m * d.r});
        }
        std::sort(regions.begin(), regions.end());
        int64_t prev = 0;
        for (auto& rg : regions) {
            CHECK(rg.first >= prev && rg.second <= plan->res_mail_slots);
            prev = rg.second;
        }
    }
    CHECK(plan->res_sync_words == kResSyncWords);
    // exactly one strip reducer per strip, one orthogonaliser per matrix, one chunk reducer per column chunk
    {
        std::vector<int> strip_red(plan->res_n_cnts, 0), chunk_red(plan->res_n_cntq, 0), ortho(plan->mats.size(), 0);
        for (const RTile& t : plan->res_tiles) {
            if (t.mat < 0) continue;
            if (t.ppart == 0) strip_red[t.cnts] += 1;
            if (t.ppart == 0 && t.row0 == 0) ortho[t.mat] += 1;
            if (t.qrun_len > 0 && t.qpart == 0) chunk_red[t.cntq] += 1;
        }
        for (int v : strip_red) CHECK(v == 1);
        for (int v : chunk_red) CHECK(v == 1);
        for (int v : ortho) CHECK(v == 1);
    }
    // every strip counter is shared by exactly the column chunks of one strip
    {
        std::vector<int> per_strip(plan->res_n_cnts, 0);
        for (const RTile& t : plan->res_tiles)
            if (t.mat >= 0) per_strip[t.cnts] += 1;
        for (const RTile& t : plan->res_tiles)
            if (t.mat >= 0) CHECK(per_strip[t.cnts] == plan->res_mats[t.mat].n_cchunk);
    }
}

static void check_p_tiling(const psgd_plan* plan) { check_cover(plan, plan->tiles1, (int)plan->tuning.k1_nv, 1); }

// Appendix G baselines: the slices of the flattened matrices (16-byte accesses: aligned starts), of the vector region
// and of the kept entries each cover their range exactly once; the packed value offsets are back to back.
static void check_baseline_tables(const psgd_plan* plan, int rank) {
    std::vector<int64_t> kept(plan->mats.size(), 0);
    int64_t kept_total = 0;
    // running slice counts: matrix i owns slices [first[i], first[i+1]), enough to cover its n m elements
    CHECK(plan->flat_first.size() == plan->mats.size() + 1 && plan->flat_first.back() == plan->flat_tiles);
    for (size_t i = 0; i < plan->mats.size(); ++i) {
        const int64_t nm = (int64_t)plan->mats[i].n * plan->mats[i].m;
        CHECK(plan->flat_first[i + 1] - plan->flat_first[i] == (nm + kFlatTileElems - 1) / kFlatTileElems);
    }
    CHECK(plan->flat_vec_tiles == (plan->sizes.n_vec_elems + kFlatTileElems - 1) / kFlatTileElems);
    CHECK((int64_t)plan->kept_slice_mat.size() == plan->kept_slices && plan->kept_slice_first.size() == plan->kept_slice_mat.size());
    for (size_t k = 0; k < plan->kept_slice_mat.size(); ++k) {
        const int32_t mi = plan->kept_slice_mat[k];
        CHECK(mi >= 0 && mi < (int)plan->mats.size() && plan->kept_slice_first[k] == kept[mi]);
        kept[mi] += std::min<int64_t>(kBlock, plan->mats[mi].kept - kept[mi]);
    }
    CHECK(plan->mat_tensor.size() == plan->mats.size());
    for (size_t i = 0; i < plan->mats.size(); ++i) {
        const MatDesc& d = plan->mats[i];
        const int64_t nm = (int64_t)d.n * d.m;
        CHECK(d.off % 4 == 0 && nm > 0);
        CHECK(d.kept == std::min<int64_t>(((int64_t)d.n + d.m) * rank, nm) && kept[i] == d.kept && d.kept_off == kept_total);
        CHECK(plan->mat_tensor[i] == d.tensor);
        kept_total += d.kept;
    }
    CHECK(kept_total == plan->sizes.kept_elems);
}

static void check_plan(const std::vector<psgd_shape>& shapes, int rank, int workers, const Tuning* tu) {
    psgd_plan* plan = nullptr;
    CHECK(psgd_plan_create(shapes.data(), (int)shapes.size(), rank, workers, PSGD_F32, PSGD_F32, &plan) == PSGD_OK);
    if (tu) {
        CHECK(psgd_plan_set_tuning(plan, "k1_rows", tu->k1_rows) == PSGD_OK);
        CHECK(psgd_plan_set_tuning(plan, "k1_nv", tu->k1_nv) == PSGD_OK);
        CHECK(psgd_plan_set_tuning(plan, "k3_rows", tu->k3_rows) == PSGD_OK);
        CHECK(psgd_plan_set_tuning(plan, "k3_nv", tu->k3_nv) == PSGD_OK);
        CHECK(psgd_plan_set_tuning(plan, "k4_rows", tu->k4_rows) == PSGD_OK);
        CHECK(psgd_plan_set_tuning(plan, "k4_nv", tu->k4_nv) == PSGD_OK);
        CHECK(psgd_plan_set_tuning(plan, "ortho_rows", tu->ortho_rows) == PSGD_OK);
    }
    check_resident(plan);
    for (int64_t rr : {5, 8, 13, 24, 32}) {
        CHECK(psgd_plan_set_tuning(plan, "res_rows", rr) == PSGD_OK);
        if (rr > res_rows_for_rank(rank)) CHECK(!plan->resident_ok);
        check_resident(plan);
    }
    CHECK(psgd_plan_set_tuning(plan, "res_rows", 0) == PSGD_OK);
    check_p_tiling(plan);
    for (int64_t xo : {0, 1, 2, 100, 2048, -1}) {   // every ordering of the tile lists for the dies covers the same elements
        CHECK(psgd_plan_set_tuning(plan, "xcd_order", xo) == PSGD_OK);
        check_cover(plan, plan->tiles1, (int)plan->tuning.k1_nv, 1);
        check_cover(plan, plan->tiles3, (int)plan->tuning.k3_nv, 2);
        check_cover(plan, plan->tiles4, (int)plan->tuning.k4_nv, 0);
        if (!plan->tiles4u.empty()) check_cover(plan, plan->tiles4u, (int)plan->tuning.k4_nv, 0);   // fused-update pass
    }
    check_cover(plan, plan->tiles3, (int)plan->tuning.k3_nv, 2);
    check_cover(plan, plan->tiles4, (int)plan->tuning.k4_nv, 0);
    // flat layout: matrices do not overlap, stay inside N, are 64-aligned
    int64_t prev_end = 0;
    for (const MatDesc& d : plan->mats) {
        CHECK(d.off % kAlignElems == 0 && d.off >= prev_end);
        prev_end = d.off + (int64_t)d.n * d.m;
        CHECK(prev_end <= plan->sizes.n_mat_elems);
        CHECK(d.r >= 1 && d.r <= rank && d.r <= d.n && d.r <= d.m);
        CHECK(d.p_off + (int64_t)d.n * d.r <= plan->sizes.p_elems);
        CHECK(d.q_off + (int64_t)d.m * d.r <= plan->sizes.q_elems);
        CHECK(d.ppart_off >= 0 && d.ppart_off + (int64_t)workers * d.n_cchunk * d.n * d.r <= plan->ws_ppart_floats);
        CHECK(d.qpart_off >= plan->ws_ppart_floats &&
              d.qpart_off + (int64_t)workers * d.n_rblock * d.m * d.r <= plan->ws_ppart_floats + plan->ws_qpart_floats);
        if ((int64_t)d.n * d.r > kPanelFloats || d.n > plan->tuning.ortho_rows) {
            CHECK(d.n_gblock == (d.n + kGramRows - 1) / kGramRows);
            CHECK(d.gram_off >= 0 && d.gram_off + (int64_t)d.n_gblock * d.r * d.r <= plan->ws_gram_doubles);
        } else {
            CHECK(d.n_gblock == 0);
        }
    }
    {
        // every matrix is orthogonalised exactly once: by one workgroup (small) or by its row blocks (tall)
        std::vector<int> small(plan->mats.size(), 0);
        std::vector<int64_t> rows(plan->mats.size(), 0);
        for (int32_t i : plan->small_mats) { CHECK(i >= 0 && i < (int)plan->mats.size()); small[i] += 1; }
        for (const Tile& t : plan->tiles_gram) {
            CHECK(t.mat >= 0 && t.mat < (int)plan->mats.size());
            const MatDesc& d = plan->mats[t.mat];
            CHECK(t.part >= 0 && t.part < d.n_gblock && t.row0 == rows[t.mat] && t.nrows > 0 && t.nrows <= kGramRows);
            rows[t.mat] += t.nrows;
        }
        for (size_t i = 0; i < plan->mats.size(); ++i) {
            const MatDesc& d = plan->mats[i];
            if (d.n_gblock == 0) CHECK(small[i] == 1 && rows[i] == 0 && (int64_t)d.n * d.r <= kPanelFloats && d.n <= plan->tuning.ortho_rows);
            else CHECK(small[i] == 0 && rows[i] == d.n);
        }
    }
    CHECK(((plan->ws_ppart_floats + plan->ws_qpart_floats) * 4 + 255) / 256 * 256 + plan->ws_gram_doubles * 8 <=
          plan->sizes.workspace_bytes);
    CHECK(plan->sizes.grad_stride >= plan->sizes.n_mat_elems + plan->sizes.n_vec_elems);
    // Q-reduction slices cover each m x r panel exactly once
    std::vector<int64_t> covered(plan->mats.size(), 0);
    for (const Tile& t : plan->tilesq) {
        CHECK(t.mat >= 0 && t.elem0 == covered[t.mat] && t.nelem > 0 && t.nelem <= kWave);
        covered[t.mat] += t.nelem;
    }
    for (size_t i = 0; i < plan->mats.size(); ++i) CHECK(covered[i] == (int64_t)plan->mats[i].m * plan->mats[i].r);
    std::vector<int64_t> covered_p(plan->mats.size(), 0);
    for (const Tile& t : plan->tilesp) {
        CHECK(t.mat >= 0 && t.elem0 == covered_p[t.mat] && t.nelem > 0 && t.nelem <= kWave);
        covered_p[t.mat] += t.nelem;
    }
    for (size_t i = 0; i < plan->mats.size(); ++i) CHECK(covered_p[i] == (int64_t)plan->mats[i].n * plan->mats[i].r);
    check_baseline_tables(plan, rank);
    psgd_plan_destroy(plan);
}

// Matrix-core path (rank > 8): every tiling covers each element once and every partial slice is in bounds.
static void check_hr_plan(const std::vector<psgd_shape>& shapes, int rank, int workers) {
    psgd_plan* plan = nullptr;
    CHECK(psgd_plan_create(shapes.data(), (int)shapes.size(), rank, workers, PSGD_F32, PSGD_F32, &plan) == PSGD_OK);
    CHECK(plan->hr && !plan->resident_ok);
    CHECK(plan->hr_nt * 16 >= rank);
    auto cover = [&](const std::vector<Tile>& tiles, bool full_rows) {
        std::vector<std::vector<unsigned char>> seen(plan->mats.size());
        for (size_t i = 0; i < plan->mats.size(); ++i) seen[i].assign((size_t)plan->mats[i].n * plan->mats[i].m, 0);
        for (const Tile& t : tiles) {
            CHECK(t.mat >= 0 && t.mat < (int)plan->mats.size());
            const MatDesc& d = plan->mats[t.mat];
            CHECK(d.m % 4 == 0 && t.row0 >= 0 && t.nrows > 0 && t.row0 + t.nrows <= d.n);
            CHECK(t.vec0 >= 0 && t.vec0 % 4 == 0 && t.nvec > 0 && t.vec0 + t.nvec <= d.m);
            if (full_rows)   // P = M Q tiles: column ranges start at multiples of 64, name their partial, bytes fit 31 bits
                CHECK(t.vec0 % 64 == 0 && t.nrows <= 256 && t.part >= 0 && t.part < d.n_cchunk &&
                      t.vec0 == (int64_t)t.part * plan->tuning.hr_k1_cols && (int64_t)t.nrows * d.m * 4 < (1LL << 31));
            else CHECK(t.nvec <= 128);
            for (int i = t.row0; i < t.row0 + t.nrows; ++i)
                for (int j = t.vec0; j < t.vec0 + t.nvec; ++j) {
                    unsigned char& sf = seen[t.mat][(size_t)i * d.m + j];
                    CHECK(sf == 0);
                    sf = 1;
                }
        }
        for (auto& v : seen)
            for (unsigned char sf : v) CHECK(sf == 1);
    };
    cover(plan->hr_tiles1, true);
    cover(plan->hr_tiles3, false);
    cover(plan->hr_tiles4, false);
    for (const Tile& t : plan->hr_tiles3) {
        const MatDesc& d = plan->mats[t.mat];
        CHECK(t.part >= 0 && t.part < d.n_rblock);
    }
    std::vector<int64_t> rows(plan->mats.size(), 0);
    for (const Tile& t : plan->tiles_gram) {
        const MatDesc& d = plan->mats[t.mat];
        CHECK(t.part >= 0 && t.part < d.n_gblock && t.row0 == rows[t.mat] && t.nrows > 0 && t.nrows <= 1024 * 1024 && d.n_gblock <= 64);
        rows[t.mat] += t.nrows;
    }
    for (size_t i = 0; i < plan->mats.size(); ++i) {
        const MatDesc& d = plan->mats[i];
        CHECK(rows[i] == d.n && d.n_cchunk == (d.m + plan->tuning.hr_k1_cols - 1) / plan->tuning.hr_k1_cols);
        CHECK(d.ppart_off >= 0 && d.ppart_off + (int64_t)workers * d.n_cchunk * d.n * d.r <= plan->ws_ppart_floats);
        CHECK(d.qpart_off >= plan->ws_ppart_floats &&
              d.qpart_off + (int64_t)workers * d.n_rblock * d.m * d.r <= plan->ws_ppart_floats + plan->ws_qpart_floats);
        CHECK(d.gram_off >= 0 && d.gram_off + (int64_t)d.n_gblock * d.r * d.r <= plan->ws_gram_doubles);
        CHECK(d.chol_off >= 0 && d.chol_off + (int64_t)d.r * d.r + d.r <= plan->ws_chol_doubles);
        CHECK(d.r <= PSGD_MAX_RANK);
    }
    CHECK(((plan->ws_ppart_floats + plan->ws_qpart_floats) * 4 + 255) / 256 * 256 +
              (plan->ws_gram_doubles + plan->ws_chol_doubles) * 8 <= plan->sizes.workspace_bytes);
    std::vector<int64_t> covered(plan->mats.size(), 0);
    for (const Tile& t : plan->tilesq) {
        CHECK(t.mat >= 0 && t.elem0 == covered[t.mat] && t.nelem > 0 && t.nelem <= kWave);
        covered[t.mat] += t.nelem;
    }
    for (size_t i = 0; i < plan->mats.size(); ++i)   // a matrix with a single partial Q needs no reduction
        CHECK(covered[i] == (workers * plan->mats[i].n_rblock > 1 ? (int64_t)plan->mats[i].m * plan->mats[i].r : 0));
    psgd_plan_destroy(plan);
}

int main() {
    std::vector<std::vector<psgd_shape>> sets = {
        {{64, 27}, {64, 576}, {64, 576}},
        {{37, 91}, {7, 1}, {50, 650}, {130, 1028}, {5, 3}, {300, 2}, {1, 40}, {1031, 1}, {3, 4700}, {257, 260}},
        {{512, 4608}, {10, 512}, {128, 64}, {9610, 1}},
        {{2600, 650}, {3328, 650}, {33280, 650}, {5000, 3}},
        {{1, 2}, {2, 1}},
        {{2048, 2048}, {2100, 2052}, {64, 27}, {3000, 1}},   // tall and wide: the taller row blocks of the second sweep
        {{37, 91}, {7, 1}, {50, 650}, {130, 1028}, {5, 3}, {300, 2}, {1, 40}, {1031, 1}, {3, 4700}, {257, 260},
         {512, 36}, {64, 27}},
        {{64, 27}, {64, 576}, {64, 576}, {64, 576}, {64, 576}, {128, 576}, {128, 1152}, {128, 1152}, {128, 1152},
         {128, 64}, {256, 1152}, {256, 2304}, {256, 2304}, {256, 2304}, {256, 128}, {512, 2304}, {512, 4608},
         {512, 4608}, {512, 4608}, {512, 256}, {10, 512}, {9610, 1}},
    };
    Tuning small;
    small.k1_rows = 8; small.k1_nv = 1; small.k3_rows = 16; small.k3_nv = 1; small.k4_rows = 8; small.k4_nv = 1;
    small.ortho_rows = kOrthoMaxRows;   // short panels by one workgroup (Gram-Schmidt in LDS)
    Tuning big;
    big.k1_rows = 64; big.k1_nv = 2; big.k3_rows = 300; big.k3_nv = 2; big.k4_rows = 300; big.k4_nv = 2;
    big.ortho_rows = 64;
    for (auto& s : sets)
        for (int rank : {1, 2, 4, 8})
            for (int W : {1, 3}) {
                check_plan(s, rank, W, nullptr);
                check_plan(s, rank, W, &small);
                check_plan(s, rank, W, &big);
            }
    {
        std::vector<psgd_shape> tr = {{1000, 256}, {256, 256}, {77, 1}, {1024, 256}, {256, 1024}, {20, 12}, {3000, 64},
                                      {130, 2308}, {64, 4096}};
        for (int rank : {9, 16, 17, 32, 64})
            for (int W : {1, 2}) check_hr_plan(tr, rank, W);
        // a row length that is not a multiple of 4 is refused on this path
        std::vector<psgd_shape> odd = {{64, 650}};
        psgd_plan* plan = nullptr;
        CHECK(psgd_plan_create(odd.data(), 1, 16, 1, PSGD_F32, PSGD_F32, &plan) == PSGD_EUNSUPPORTED);
        // bf16 data at rank <= 8 run on the streaming kernels at any row length; the matrix-core kernels refuse it
        CHECK(psgd_plan_create(odd.data(), 1, 4, 1, PSGD_BF16, PSGD_F32, &plan) == PSGD_OK);
        CHECK(psgd_plan_set_tuning(plan, "bf16_valu", 0) == PSGD_EUNSUPPORTED);
        CHECK(!plan->hr);
        psgd_plan_destroy(plan);
    }
    std::printf("OK\n");
    return 0;
}
