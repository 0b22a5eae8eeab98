// Calibration Hessian  H += scale * X X^T  (Section 3.1, "Saliency scores and weight update";
// factor 2 per the caption of Algorithm 1 is the caller's `scale`).
//
// A symmetric rank-n_tok update on the fp32 matrix cores: only the lower-triangular list of
// 128 x 128 output tiles is computed; every strictly-lower tile is also written transposed, so both
// triangles of H are valid.  When the triangular tile list alone cannot fill the chip the token
// range is split; the splits write raw accumulators to the workspace and count themselves at their tile, and the
// one that counts last adds all sets in split order (fixed summation order whoever is last: results do not change
// from run to run) and applies the epilogue.
#include "common.h"
#include "mfma_gemm.h"

namespace ziplm {

// compute units of the current device (cached per device; concurrent first calls store the same value)
int device_cu_count() {
    constexpr int kMaxDevices = 64;
    static int cached[kMaxDevices] = {};
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;   // MI355X; used only for sizing when no device is visible
    if (dev >= 0 && dev < kMaxDevices && cached[dev] > 0) return cached[dev];
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
    if (dev >= 0 && dev < kMaxDevices) cached[dev] = n;
    return n;
}

// Slices of 32 tokens between two carry-overs of the matrix-core accumulators into the second accumulator set:
// chains of 128 matrix instructions, whose rounding is 2e-7 of a 256-token chunk sum and averages out over the
// chunks.  The second set takes one rounding per chunk, so a workgroup gets at most 64 chunks (16384 tokens).
constexpr int HESSIAN_CHUNK = 8;
constexpr int64_t HESSIAN_MAX_TOKENS_PER_SPLIT = 64 * HESSIAN_CHUNK * gemm::BK;

struct HessianPlan {
    int tiles;        // lower-triangular tile count
    int nsplit;       // token splits
    int64_t k_chunk;  // tokens per split (multiple of 32)
    size_t ws_bytes, partial_bytes;
};

static HessianPlan plan_hessian(int d_col, int64_t n_tok) {
    HessianPlan p;
    const int tm = (d_col + gemm::BM - 1) / gemm::BM;
    p.tiles = tm * (tm + 1) / 2;
    const int slots = 2 * device_cu_count();  // two workgroups fit per compute unit
    // Pick the split count that fills whole rounds of `slots` workgroups best, keeping at least
    // 512 tokens per split; prefer fewer splits when the gain is below 3%.
    const int min_split = (int)((n_tok + HESSIAN_MAX_TOKENS_PER_SPLIT - 1) / HESSIAN_MAX_TOKENS_PER_SPLIT);
    int best = min_split;
    double best_eff = 0.0;
    int64_t max_split = n_tok / 512 > 0 ? (n_tok / 512 < 64 ? n_tok / 512 : 64) : 1;
    if (max_split < min_split) max_split = min_split;
    for (int s = min_split; s <= (int)max_split; ++s) {
        const int64_t blocks = (int64_t)p.tiles * s;
        const int64_t rounds = (blocks + slots - 1) / slots;
        const double eff = (double)blocks / (double)(rounds * slots);
        if (eff > best_eff * 1.03) { best_eff = eff; best = s; }
    }
    p.nsplit = best;
    int64_t chunk = (n_tok + best - 1) / best;
    chunk = (chunk + gemm::BK - 1) / gemm::BK * gemm::BK;
    p.k_chunk = chunk > 0 ? chunk : gemm::BK;
    p.nsplit = (int)((n_tok + p.k_chunk - 1) / p.k_chunk);
    if (p.nsplit < 1) p.nsplit = 1;
    // accumulator sets of the splits, then one arrival counter per tile
    p.partial_bytes = p.nsplit > 1 ? align_up((size_t)p.nsplit * p.tiles * 64 * gemm::THREADS * sizeof(float)) : 0;
    p.ws_bytes = p.nsplit > 1 ? p.partial_bytes + align_up(sizeof(int) * (size_t)p.tiles) : 0;
    return p;
}

template <int MODE, bool VEC>
static int run_hessian(const gemm::Args &base, const HessianPlan &plan, hipStream_t stream) {
    gemm::Args g = base;
    if (plan.nsplit == 1) {
        hipLaunchKernelGGL((gemm::gemm_kernel<MODE, MODE, VEC, true, false, HESSIAN_CHUNK>), dim3(plan.tiles, 1, 1),
                           dim3(gemm::THREADS), 0, stream, g);
        ZIPLM_HIP_TRY(hipGetLastError());
        return ZIPLM_OK;
    }
    // the splits count themselves at their tile; the one that counts last adds all sets in split order (one launch)
    g.flags |= gemm::F_PARTIAL;
    if (zero_fill(g.tile_counters, plan.ws_bytes - plan.partial_bytes, stream) != ZIPLM_OK) return ZIPLM_ERR_DEVICE;
    hipLaunchKernelGGL((gemm::gemm_kernel<MODE, MODE, VEC, true, false, HESSIAN_CHUNK, true>), dim3(plan.tiles, plan.nsplit, 1),
                       dim3(gemm::THREADS), 0, stream, g);
    ZIPLM_HIP_TRY(hipGetLastError());
    return ZIPLM_OK;
}

}  // namespace ziplm

extern "C" size_t ziplm_hessian_workspace_bytes(int d_col, int64_t n_tok) {
    if (d_col <= 0 || n_tok <= 0) return 0;
    return ziplm::plan_hessian(d_col, n_tok).ws_bytes;
}

extern "C" int ziplm_hessian_accumulate(float *H, const float *X, int d_col, int64_t n_tok, int64_t ldx,
                                        int layout, float scale, void *workspace, size_t workspace_bytes,
                                        void *stream) {
    using namespace ziplm;
    if (!H || d_col <= 0 || n_tok < 0) return ZIPLM_ERR_INVALID_ARG;
    if (layout != ZIPLM_X_FEATURE_MAJOR && layout != ZIPLM_X_TOKEN_MAJOR) return ZIPLM_ERR_INVALID_ARG;
    if (n_tok == 0) return ZIPLM_OK;
    if (!X) return ZIPLM_ERR_INVALID_ARG;
    if (layout == ZIPLM_X_FEATURE_MAJOR ? ldx < n_tok : ldx < d_col) return ZIPLM_ERR_INVALID_ARG;
    const HessianPlan plan = plan_hessian(d_col, n_tok);
    if (!workspace_ok(workspace, workspace_bytes, plan.ws_bytes)) return ZIPLM_ERR_WORKSPACE;

    gemm::Args g = {};
    g.A = X; g.B = X; g.C = H;
    g.M = d_col; g.N = d_col; g.K = n_tok;
    g.lda = ldx; g.ldb = ldx; g.ldc = d_col;
    g.alpha = scale; g.beta = 1.0f;
    g.flags = gemm::F_TRI_GRID | gemm::F_MIRROR;
    g.k_chunk = plan.k_chunk;
    g.partial = static_cast<float *>(workspace);
    g.tile_counters = plan.nsplit > 1 ? reinterpret_cast<int *>(static_cast<char *>(workspace) + plan.partial_bytes) : nullptr;
    g.tiles_n = (d_col + gemm::BN - 1) / gemm::BN;
    const bool vec = (ldx % 4 == 0) && (reinterpret_cast<uintptr_t>(X) % 16 == 0);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (layout == ZIPLM_X_FEATURE_MAJOR)
        return vec ? run_hessian<gemm::K_CONTIG, true>(g, plan, st) : run_hessian<gemm::K_CONTIG, false>(g, plan, st);
    return vec ? run_hessian<gemm::R_CONTIG, true>(g, plan, st) : run_hessian<gemm::R_CONTIG, false>(g, plan, st);
}
