// C ABI of libtbik: argument validation, variant choice, launches.  No device memory is allocated here.
#include <atomic>

#include "tbik_internal.hpp"

using namespace tbik;

namespace {

std::atomic<int> g_last_hip_error{0};
std::atomic<int> g_forced_variant{VARIANT_AUTO};

const char *const kVariantNames[VARIANT_COUNT] = {"auto", "reference", "tile128x128", "tile32x128", "tile64x128"};

inline bool is_pow2(int64_t v) { return v >= 1 && (v & (v - 1)) == 0; }
inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int hip_fail(hipError_t e) {
    g_last_hip_error.store((int)e);
    return TBIK_ERR_HIP;
}

// Shape rules common to the GEMM entry points; fills superleaf / ns.
int check_tree(int M, int N, int K, int leaf, int k_first, int P, int *superleaf, int *ns) {
    if (M < 0 || N < 0 || K <= 0 || leaf <= 0 || k_first < 0) return TBIK_ERR_SHAPE;
    if (k_first == 0) {                       // the smallest legal choice: the odd part of the number of leaves
        if (K % leaf != 0) return TBIK_ERR_SHAPE;
        int64_t q = K / leaf;
        while (q % 2 == 0) q /= 2;
        k_first = (int)q;
    }
    const int64_t sl = (int64_t)leaf * k_first;
    if (sl > K || K % sl != 0 || sl % 16 != 0) return TBIK_ERR_SHAPE;
    const int64_t n = K / sl;
    if (!is_pow2(n)) return TBIK_ERR_SHAPE;
    if (P < 1 || !is_pow2(P) || P > n || P > TBIK_MAX_SHARDS) return TBIK_ERR_SHARDS;
    *superleaf = (int)sl;
    *ns = (int)n;
    return TBIK_OK;
}

int check_operands(int x_dtype, const void *X, int64_t ldx, const void *W, int64_t ldw, int N, int K) {
    if (!X || !W) return TBIK_ERR_NULL;
    if (ldx < K || ldw < N) return TBIK_ERR_SHAPE;
    const int per16 = (x_dtype == TBIK_F32) ? 4 : 8;       // elements per 16 bytes
    if (!aligned(X, 16) || !aligned(W, 16) || ldx % per16 != 0 || ldw % per16 != 0) return TBIK_ERR_ALIGN;
    return TBIK_OK;
}

// The kernels of an operand format.
bool tiled_supports(const GemmArgs &a, int variant) {
    return a.x_dtype == TBIK_F32 ? gemm_f32_tiled_supports(a) : gemm_tiled_supports(a, variant);
}
hipError_t launch_reference(const GemmArgs &a, hipStream_t s) {
    return a.x_dtype == TBIK_F32 ? launch_gemm_f32_reference(a, s) : launch_gemm_reference(a, s);
}
hipError_t launch_tiled(const GemmArgs &a, int variant, hipStream_t s) {
    return a.x_dtype == TBIK_F32 ? launch_gemm_f32_tiled(a, variant, s) : launch_gemm_tiled(a, variant, s);
}

// Rows of the workgroup tile for a shape (pure): 32 for M <= 32, 64 for M <= 64, else 128 -- unless the 128-row tiles
// would leave a quarter or more of the compute units without one while the 64-row tiles fill exactly one round: then
// 64, which spares the K split (a second launch and an fp32 round trip of the partial sums).  Measured: o_proj
// M = 512 30.6 -> 24.1 us, down_proj M = 512 72.7 -> 61.5 us; with two ragged rounds of 64-row tiles it loses.
int tile_rows(int M, int N) {
    if (M <= 32) return 32;
    if (M <= 64) return 64;
    const int64_t cols = ((int64_t)N + 127) / 128;
    const int64_t tiles128 = (((int64_t)M + 127) / 128) * cols, tiles64 = (((int64_t)M + 63) / 64) * cols;
    return (tiles128 < 192 && tiles64 >= 192 && tiles64 <= 256) ? 64 : 128;
}

// Internal split of K across workgroups (a pure function of the shape, so that tbik_gemm_workspace_bytes() can be
// evaluated without a device): the kernel is launched as if the caller had asked for `split` shards (fp32 partials into
// the workspace) and the partials are combined by the same tree (Theorem 1: identical bits).  Reasons to split: a
// register-resident tree of more than 16 superleaves; fewer than 128 tiles (most compute units idle); and, for very
// long K, rounds -- 256 compute units take the work items in rounds, so 320 tiles cost two rounds of whole-K tiles
// unsplit but five rounds of quarter-K items split in four (32B-class down_proj, K = 25600: M = 1024 454 -> 323 us,
// M = 512 218 -> 189 us, M = 128 78 -> 64 us).  The price of a split is the partials' round trip, the second launch and
// a pipeline fill per item; at K <= 12288 splitting for rounds measured slower (o_proj M = 768: 31 -> 46 us), so there
// only the first two reasons apply.
int internal_split(int M, int N, int K, int ns) {
    const int64_t bm = tile_rows(M, N);
    const int64_t tiles = ((M + bm - 1) / bm) * (((int64_t)N + 127) / 128);
    int split = 1;
    while (ns / split > 16 && split < TBIK_MAX_SHARDS) split *= 2;   // the tiled kernel walks at most 16 superleaves per shard
    if (K >= 16384) {
        int best = split;
        double best_cost = 0;
        for (int s = split; s <= ns && s <= 16; s *= 2) {
            const double rounds = (double)((tiles * s + 255) / 256);
            const double cost = rounds / s + (s > 1 ? 0.015 + 0.005 * s : 0.0);
            if (s == split || cost < best_cost - 1e-9) { best = s; best_cost = cost; }
        }
        return best;
    }
    if (tiles >= 128) return split;             // at least half of the 256 compute units already have a tile
    while (split < ns && split < 16 && tiles * split < 256) split *= 2;
    return split;
}

int pick_variant(const GemmArgs &a) {
    const int forced = g_forced_variant.load();
    if (forced != VARIANT_AUTO) return (forced == VARIANT_REFERENCE || tiled_supports(a, forced)) ? forced : VARIANT_REFERENCE;
    if (a.x_dtype == TBIK_F32) return gemm_f32_tiled_supports(a) ? VARIANT_AUTO : VARIANT_REFERENCE;    // the launcher picks the tile
    const int rows = tile_rows(a.M, a.N);
    if (rows == 128 && gemm_tiled_supports(a, VARIANT_T128)) return VARIANT_T128;
    if (rows >= 64 && gemm_tiled_supports(a, VARIANT_T64)) return VARIANT_T64;
    if (gemm_tiled_supports(a, VARIANT_T32)) return VARIANT_T32;
    if (gemm_tiled_supports(a, VARIANT_T128)) return VARIANT_T128;
    return VARIANT_REFERENCE;
}

// 16-bit output type that goes with an operand format.
inline bool legal_y_dtype(int y_dtype, int x_dtype) { return y_dtype == TBIK_F32 || y_dtype == x_dtype; }

}  // namespace

extern "C" {

size_t tbik_gemm_workspace_bytes(int M, int N, int K, int leaf, int k_first) {
    int sl, ns;
    if (check_tree(M, N, K, leaf, k_first, 1, &sl, &ns) != TBIK_OK) return 0;
    // fp32 partials of the internal K split, if this shape uses one
    const int split = internal_split(M, N, K, ns);
    return split > 1 ? (size_t)split * (size_t)M * (size_t)N * sizeof(float) : 0;
}

}  // extern "C"

namespace {

int gemm_shard_partials(int x_dtype, const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                        int M, int N, int K, int leaf, int k_first, int P, void *hip_stream) {
    int sl, ns;
    int rc = check_tree(M, N, K, leaf, k_first, P, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (M == 0 || N == 0) return TBIK_OK;
    rc = check_operands(x_dtype, X, ldx, W, ldw, N, K);
    if (rc != TBIK_OK) return rc;
    if (!partials) return TBIK_ERR_NULL;
    if (!aligned(partials, 16)) return TBIK_ERR_ALIGN;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)W, ldw, partials, nullptr, 0, TBIK_F32, M, N, K, sl, ns, P, x_dtype};
    hipStream_t s = (hipStream_t)hip_stream;
    const int v = pick_variant(a);
    hipError_t e = (v == VARIANT_REFERENCE) ? launch_reference(a, s) : launch_tiled(a, v, s);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int gemm(int x_dtype, const void *X, int64_t ldx, const void *W, int64_t ldw, void *Y, int64_t ldy,
         int y_dtype, int M, int N, int K, int leaf, int k_first,
         void *workspace, size_t workspace_bytes, void *hip_stream) {
    int sl, ns;
    int rc = check_tree(M, N, K, leaf, k_first, 1, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (!legal_y_dtype(y_dtype, x_dtype)) return TBIK_ERR_DTYPE;
    if (M == 0 || N == 0) return TBIK_OK;
    rc = check_operands(x_dtype, X, ldx, W, ldw, N, K);
    if (rc != TBIK_OK) return rc;
    if (!Y) return TBIK_ERR_NULL;
    if (ldy < N) return TBIK_ERR_SHAPE;
    if (!aligned(Y, y_dtype == TBIK_F32 ? 4 : 2)) return TBIK_ERR_ALIGN;
    const size_t need = tbik_gemm_workspace_bytes(M, N, K, leaf, k_first);
    if (need > 0 && (!workspace || workspace_bytes < need)) return TBIK_ERR_WORKSPACE;
    if (workspace && !aligned(workspace, 256)) return TBIK_ERR_ALIGN;

    hipStream_t s = (hipStream_t)hip_stream;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)W, ldw, nullptr, Y, ldy, y_dtype, M, N, K, sl, ns, 1, x_dtype};
    const int split = internal_split(M, N, K, ns);
    GemmArgs probe = a;
    probe.P = split;
    const int v = pick_variant(probe);
    hipError_t e;
    if (split == 1 || v == VARIANT_REFERENCE) {
        e = (v == VARIANT_REFERENCE) ? launch_reference(a, s) : launch_tiled(a, v, s);
    } else {
        a.partials = reinterpret_cast<float *>(workspace);
        a.Y = nullptr;
        a.P = split;
        e = launch_tiled(a, v, s);
        if (e == hipSuccess) e = launch_tree_combine(a.partials, split, Y, ldy, y_dtype, M, N, s);
    }
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int gemm_reference(int x_dtype, const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                   void *Y, int64_t ldy, int y_dtype,
                   int M, int N, int K, int leaf, int k_first, int P, void *hip_stream) {
    int sl, ns;
    int rc = check_tree(M, N, K, leaf, k_first, P, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (!legal_y_dtype(y_dtype, x_dtype)) return TBIK_ERR_DTYPE;
    if (M == 0 || N == 0) return TBIK_OK;
    rc = check_operands(x_dtype, X, ldx, W, ldw, N, K);
    if (rc != TBIK_OK) return rc;
    if (!partials && !Y) return TBIK_ERR_NULL;
    if (Y && P != 1) return TBIK_ERR_SHARDS;
    if (Y && ldy < N) return TBIK_ERR_SHAPE;
    if (Y && !aligned(Y, y_dtype == TBIK_F32 ? 4 : 2)) return TBIK_ERR_ALIGN;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)W, ldw, partials, Y, ldy, y_dtype, M, N, K, sl, ns, P, x_dtype};
    hipError_t e = launch_reference(a, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

}  // namespace

extern "C" {

int tbik_gemm(const void *X, int64_t ldx, const void *W, int64_t ldw, void *Y, int64_t ldy,
              tbik_dtype y_dtype, int M, int N, int K, int leaf, int k_first,
              void *workspace, size_t workspace_bytes, void *hip_stream) {
    return gemm(TBIK_BF16, X, ldx, W, ldw, Y, ldy, (int)y_dtype, M, N, K, leaf, k_first, workspace, workspace_bytes, hip_stream);
}

int tbik_gemm_f16(const void *X, int64_t ldx, const void *W, int64_t ldw, void *Y, int64_t ldy,
                  tbik_dtype y_dtype, int M, int N, int K, int leaf, int k_first,
                  void *workspace, size_t workspace_bytes, void *hip_stream) {
    return gemm(TBIK_F16, X, ldx, W, ldw, Y, ldy, (int)y_dtype, M, N, K, leaf, k_first, workspace, workspace_bytes, hip_stream);
}

int tbik_gemm_shard_partials(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                             int M, int N, int K, int leaf, int k_first, int P,
                             void *workspace, size_t workspace_bytes, void *hip_stream) {
    (void)workspace; (void)workspace_bytes;
    return gemm_shard_partials(TBIK_BF16, X, ldx, W, ldw, partials, M, N, K, leaf, k_first, P, hip_stream);
}

int tbik_gemm_shard_partials_f16(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                                 int M, int N, int K, int leaf, int k_first, int P,
                                 void *workspace, size_t workspace_bytes, void *hip_stream) {
    (void)workspace; (void)workspace_bytes;
    return gemm_shard_partials(TBIK_F16, X, ldx, W, ldw, partials, M, N, K, leaf, k_first, P, hip_stream);
}

int tbik_gemm_reference(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                        void *Y, int64_t ldy, tbik_dtype y_dtype,
                        int M, int N, int K, int leaf, int k_first, int P, void *hip_stream) {
    return gemm_reference(TBIK_BF16, X, ldx, W, ldw, partials, Y, ldy, (int)y_dtype, M, N, K, leaf, k_first, P, hip_stream);
}

int tbik_gemm_reference_f16(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                            void *Y, int64_t ldy, tbik_dtype y_dtype,
                            int M, int N, int K, int leaf, int k_first, int P, void *hip_stream) {
    return gemm_reference(TBIK_F16, X, ldx, W, ldw, partials, Y, ldy, (int)y_dtype, M, N, K, leaf, k_first, P, hip_stream);
}

int tbik_gemm_f32(const void *X, int64_t ldx, const void *W, int64_t ldw, void *Y, int64_t ldy,
                  int M, int N, int K, int leaf, int k_first,
                  void *workspace, size_t workspace_bytes, void *hip_stream) {
    return gemm(TBIK_F32, X, ldx, W, ldw, Y, ldy, TBIK_F32, M, N, K, leaf, k_first, workspace, workspace_bytes, hip_stream);
}

int tbik_gemm_shard_partials_f32(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                                 int M, int N, int K, int leaf, int k_first, int P,
                                 void *workspace, size_t workspace_bytes, void *hip_stream) {
    (void)workspace; (void)workspace_bytes;
    return gemm_shard_partials(TBIK_F32, X, ldx, W, ldw, partials, M, N, K, leaf, k_first, P, hip_stream);
}

int tbik_gemm_reference_f32(const void *X, int64_t ldx, const void *W, int64_t ldw, float *partials,
                            void *Y, int64_t ldy, int M, int N, int K, int leaf, int k_first, int P, void *hip_stream) {
    return gemm_reference(TBIK_F32, X, ldx, W, ldw, partials, Y, ldy, TBIK_F32, M, N, K, leaf, k_first, P, hip_stream);
}

int tbik_tree_combine(const float *partials, int P, void *Y, int64_t ldy, tbik_dtype y_dtype,
                      int M, int N, void *hip_stream) {
    if (M < 0 || N < 0) return TBIK_ERR_SHAPE;
    if (P < 1 || !is_pow2(P) || P > TBIK_MAX_SHARDS) return TBIK_ERR_SHARDS;
    if (y_dtype != TBIK_F32 && y_dtype != TBIK_BF16 && y_dtype != TBIK_F16) return TBIK_ERR_DTYPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!partials || !Y) return TBIK_ERR_NULL;
    if (ldy < N) return TBIK_ERR_SHAPE;
    if (!aligned(partials, 16) || !aligned(Y, y_dtype == TBIK_F32 ? 4 : 2)) return TBIK_ERR_ALIGN;
    hipError_t e = launch_tree_combine(partials, P, Y, ldy, (int)y_dtype, M, N, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

// ---- 8-bit floating-point operands ----
static bool is_fp8(int d) { return d == TBIK_FP8_E4M3 || d == TBIK_FP8_E5M2; }

// Rows of the 8-bit kernel's workgroup tile: the rule of the 16-bit kernels, or what tbik_set_gemm_variant forces.
static int fp8_tile_rows(int M, int N) {
    switch (g_forced_variant.load()) {
        case VARIANT_T128: return 128;
        case VARIANT_T64: return 64;
        case VARIANT_T32: return 32;
        default: return tile_rows(M, N);
    }
}

static int fp8_checks(int x_dtype, const void *X, int64_t ldx, const void *Wt, int64_t ldwt, int M, int N, int K,
                      int leaf, int k_first, int P, int *sl, int *ns) {
    int rc = check_tree(M, N, K, leaf, k_first, P, sl, ns);
    if (rc != TBIK_OK) return rc;
    if (!is_fp8(x_dtype)) return TBIK_ERR_DTYPE;
    if (*sl % 64 != 0) return TBIK_ERR_SHAPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!X || !Wt) return TBIK_ERR_NULL;
    if (ldx < K || ldwt < K) return TBIK_ERR_SHAPE;
    if (!aligned(X, 16) || !aligned(Wt, 16) || ldx % 16 != 0 || ldwt % 16 != 0) return TBIK_ERR_ALIGN;
    return TBIK_OK;
}

size_t tbik_gemm_fp8_workspace_bytes(int M, int N, int K, int leaf, int k_first) {
    int sl, ns;
    if (check_tree(M, N, K, leaf, k_first, 1, &sl, &ns) != TBIK_OK) return 0;
    const int split = internal_split(M, N, K, ns);         // the tile shapes and the rule of the 16-bit kernels
    return split > 1 ? (size_t)split * (size_t)M * (size_t)N * sizeof(float) : 0;
}

int tbik_gemm_fp8(const void *X, int64_t ldx, const void *Wt, int64_t ldwt, void *Y, int64_t ldy,
                  tbik_dtype y_dtype, tbik_dtype x_dtype, int M, int N, int K, int leaf, int k_first,
                  void *workspace, size_t workspace_bytes, void *hip_stream) {
    int sl, ns;
    int rc = fp8_checks((int)x_dtype, X, ldx, Wt, ldwt, M, N, K, leaf, k_first, 1, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (y_dtype != TBIK_F32 && y_dtype != TBIK_BF16) return TBIK_ERR_DTYPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!Y) return TBIK_ERR_NULL;
    if (ldy < N) return TBIK_ERR_SHAPE;
    if (!aligned(Y, y_dtype == TBIK_F32 ? 4 : 2)) return TBIK_ERR_ALIGN;
    const size_t need = tbik_gemm_fp8_workspace_bytes(M, N, K, leaf, k_first);
    if (need > 0 && (!workspace || workspace_bytes < need)) return TBIK_ERR_WORKSPACE;
    if (workspace && !aligned(workspace, 256)) return TBIK_ERR_ALIGN;
    hipStream_t s = (hipStream_t)hip_stream;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, nullptr, Y, ldy, (int)y_dtype, M, N, K, sl, ns, 1, (int)x_dtype, 0};
    const int split = internal_split(M, N, K, ns);
    const int rows = fp8_tile_rows(M, N);
    GemmArgs probe = a;
    probe.P = split;
    const bool tiled = g_forced_variant.load() != VARIANT_REFERENCE && gemm_fp8_tiled_supports(probe);
    hipError_t e;
    if (!tiled) {
        e = launch_gemm_fp8_reference(a, s);
    } else if (split == 1) {
        e = launch_gemm_fp8_tiled(a, rows, s);
    } else {
        a.partials = reinterpret_cast<float *>(workspace);
        a.Y = nullptr;
        a.P = split;
        e = launch_gemm_fp8_tiled(a, rows, s);
        if (e == hipSuccess) e = launch_tree_combine(a.partials, split, Y, ldy, (int)y_dtype, M, N, s);
    }
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_gemm_shard_partials_fp8(const void *X, int64_t ldx, const void *Wt, int64_t ldwt, float *partials,
                                 tbik_dtype x_dtype, int M, int N, int K, int leaf, int k_first, int P,
                                 void *workspace, size_t workspace_bytes, void *hip_stream) {
    (void)workspace; (void)workspace_bytes;
    int sl, ns;
    int rc = fp8_checks((int)x_dtype, X, ldx, Wt, ldwt, M, N, K, leaf, k_first, P, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!partials) return TBIK_ERR_NULL;
    if (!aligned(partials, 16)) return TBIK_ERR_ALIGN;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, partials, nullptr, 0, TBIK_F32, M, N, K, sl, ns, P, (int)x_dtype, 0};
    const bool tiled = g_forced_variant.load() != VARIANT_REFERENCE && gemm_fp8_tiled_supports(a);
    hipError_t e = tiled ? launch_gemm_fp8_tiled(a, fp8_tile_rows(M, N), (hipStream_t)hip_stream)
                         : launch_gemm_fp8_reference(a, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_gemm_reference_fp8(const void *X, int64_t ldx, const void *Wt, int64_t ldwt, float *partials,
                            void *Y, int64_t ldy, tbik_dtype y_dtype, tbik_dtype x_dtype,
                            int M, int N, int K, int leaf, int k_first, int P, void *hip_stream) {
    int sl, ns;
    int rc = fp8_checks((int)x_dtype, X, ldx, Wt, ldwt, M, N, K, leaf, k_first, P, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (y_dtype != TBIK_F32 && y_dtype != TBIK_BF16) return TBIK_ERR_DTYPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!partials && !Y) return TBIK_ERR_NULL;
    if (Y && P != 1) return TBIK_ERR_SHARDS;
    if (Y && ldy < N) return TBIK_ERR_SHAPE;
    if (Y && !aligned(Y, y_dtype == TBIK_F32 ? 4 : 2)) return TBIK_ERR_ALIGN;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, partials, Y, ldy, (int)y_dtype, M, N, K, sl, ns, P, (int)x_dtype, 0};
    hipError_t e = launch_gemm_fp8_reference(a, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

// ---- MXFP4 operands ----
static int mxfp4_checks(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                        const void *Ws, int64_t ldws, int M, int N, int K, int leaf, int k_first, int P, int *sl, int *ns) {
    int rc = check_tree(M, N, K, leaf, k_first, P, sl, ns);
    if (rc != TBIK_OK) return rc;
    if (*sl % 64 != 0) return TBIK_ERR_SHAPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!X || !Wt || !Xs || !Ws) return TBIK_ERR_NULL;
    if (ldx < K / 2 || ldwt < K / 2 || ldxs < K / 32 || ldws < K / 32) return TBIK_ERR_SHAPE;
    if (!aligned(X, 16) || !aligned(Wt, 16) || ldx % 16 != 0 || ldwt % 16 != 0) return TBIK_ERR_ALIGN;
    return TBIK_OK;
}

// From 128 rows on the microscaling GEMMs re-tile their scales first (a launch of its own, which a small batch would
// feel): the workspace is the fp32 planes of the K split, rounded up to 256 bytes, then the re-tiled scales.
static bool mx_retiles(int M) { return M >= 128; }
static size_t mx_planes_bytes(int M, int N, int K, int leaf, int k_first) {
    return (tbik_gemm_fp8_workspace_bytes(M, N, K, leaf, k_first) + 255) & ~(size_t)255;      // the same tile shapes, the same K split
}
size_t tbik_gemm_mxfp4_workspace_bytes(int M, int N, int K, int leaf, int k_first) {
    int sl, ns;
    if (check_tree(M, N, K, leaf, k_first, 1, &sl, &ns) != TBIK_OK) return 0;
    return mx_planes_bytes(M, N, K, leaf, k_first) + (mx_retiles(M) && K % 256 == 0 ? mxfp4_retiled_scales_bytes(M, N, K) : 0);
}

int tbik_gemm_mxfp4(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                    const void *Ws, int64_t ldws, void *Y, int64_t ldy, tbik_dtype y_dtype,
                    int M, int N, int K, int leaf, int k_first,
                    void *workspace, size_t workspace_bytes, void *hip_stream) {
    int sl, ns;
    int rc = mxfp4_checks(X, ldx, Xs, ldxs, Wt, ldwt, Ws, ldws, M, N, K, leaf, k_first, 1, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (y_dtype != TBIK_F32 && y_dtype != TBIK_BF16) return TBIK_ERR_DTYPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!Y) return TBIK_ERR_NULL;
    if (ldy < N) return TBIK_ERR_SHAPE;
    if (!aligned(Y, y_dtype == TBIK_F32 ? 4 : 2)) return TBIK_ERR_ALIGN;
    const size_t need = tbik_gemm_mxfp4_workspace_bytes(M, N, K, leaf, k_first);
    if (need > 0 && (!workspace || workspace_bytes < need)) return TBIK_ERR_WORKSPACE;
    if (workspace && !aligned(workspace, 256)) return TBIK_ERR_ALIGN;
    hipStream_t s = (hipStream_t)hip_stream;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, nullptr, Y, ldy, (int)y_dtype, M, N, K, sl, ns, 1, TBIK_MXFP4, 0};
    const Mxfp4Scales sc{(const uint8_t *)Xs, ldxs, (const uint8_t *)Ws, ldws};
    const int split = internal_split(M, N, K, ns);
    const int rows = fp8_tile_rows(M, N);
    GemmArgs probe = a;
    probe.P = split;
    const bool tiled = g_forced_variant.load() != VARIANT_REFERENCE && gemm_mxfp4_tiled_supports(probe, sc);
    hipError_t e;
    void *retiled = (tiled && mx_retiles(M)) ? static_cast<char *>(workspace) + mx_planes_bytes(M, N, K, leaf, k_first) : nullptr;
    if (!tiled) {
        e = launch_gemm_mxfp4_reference(a, sc, s);
    } else if (split == 1) {
        e = launch_gemm_mxfp4_tiled(a, sc, rows, retiled, s);
    } else {
        a.partials = reinterpret_cast<float *>(workspace);
        a.Y = nullptr;
        a.P = split;
        e = launch_gemm_mxfp4_tiled(a, sc, rows, retiled, s);
        if (e == hipSuccess) e = launch_tree_combine(a.partials, split, Y, ldy, (int)y_dtype, M, N, s);
    }
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_gemm_shard_partials_mxfp4(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                                   const void *Ws, int64_t ldws, float *partials,
                                   int M, int N, int K, int leaf, int k_first, int P,
                                   void *workspace, size_t workspace_bytes, void *hip_stream) {
    int sl, ns;
    int rc = mxfp4_checks(X, ldx, Xs, ldxs, Wt, ldwt, Ws, ldws, M, N, K, leaf, k_first, P, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!partials) return TBIK_ERR_NULL;
    if (!aligned(partials, 16)) return TBIK_ERR_ALIGN;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, partials, nullptr, 0, TBIK_F32, M, N, K, sl, ns, P, TBIK_MXFP4, 0};
    const Mxfp4Scales sc{(const uint8_t *)Xs, ldxs, (const uint8_t *)Ws, ldws};
    const bool tiled = g_forced_variant.load() != VARIANT_REFERENCE && gemm_mxfp4_tiled_supports(a, sc);
    // a workspace as tbik_gemm_mxfp4 takes it has room for the re-tiled scales behind the planes of the K cut
    void *retiled = (tiled && mx_retiles(M) && workspace && aligned(workspace, 256) &&
                     workspace_bytes >= tbik_gemm_mxfp4_workspace_bytes(M, N, K, leaf, k_first))
                        ? static_cast<char *>(workspace) + mx_planes_bytes(M, N, K, leaf, k_first) : nullptr;
    hipError_t e = tiled ? launch_gemm_mxfp4_tiled(a, sc, fp8_tile_rows(M, N), retiled, (hipStream_t)hip_stream)
                         : launch_gemm_mxfp4_reference(a, sc, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_gemm_reference_mxfp4(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                              const void *Ws, int64_t ldws, float *partials, void *Y, int64_t ldy, tbik_dtype y_dtype,
                              int M, int N, int K, int leaf, int k_first, int P, void *hip_stream) {
    int sl, ns;
    int rc = mxfp4_checks(X, ldx, Xs, ldxs, Wt, ldwt, Ws, ldws, M, N, K, leaf, k_first, P, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (y_dtype != TBIK_F32 && y_dtype != TBIK_BF16) return TBIK_ERR_DTYPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!partials && !Y) return TBIK_ERR_NULL;
    if (Y && P != 1) return TBIK_ERR_SHARDS;
    if (Y && ldy < N) return TBIK_ERR_SHAPE;
    if (Y && !aligned(Y, y_dtype == TBIK_F32 ? 4 : 2)) return TBIK_ERR_ALIGN;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, partials, Y, ldy, (int)y_dtype, M, N, K, sl, ns, P, TBIK_MXFP4, 0};
    const Mxfp4Scales sc{(const uint8_t *)Xs, ldxs, (const uint8_t *)Ws, ldws};
    hipError_t e = launch_gemm_mxfp4_reference(a, sc, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

// ---- MXFP8 operands ----
static int mxfp8_checks(int x_dtype, const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                        const void *Ws, int64_t ldws, int M, int N, int K, int leaf, int k_first, int P, int *sl, int *ns) {
    int rc = fp8_checks(x_dtype, X, ldx, Wt, ldwt, M, N, K, leaf, k_first, P, sl, ns);
    if (rc != TBIK_OK) return rc;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!Xs || !Ws) return TBIK_ERR_NULL;
    if (ldxs < K / 32 || ldws < K / 32) return TBIK_ERR_SHAPE;
    return TBIK_OK;
}

size_t tbik_gemm_mxfp8_workspace_bytes(int M, int N, int K, int leaf, int k_first) {
    int sl, ns;
    if (check_tree(M, N, K, leaf, k_first, 1, &sl, &ns) != TBIK_OK) return 0;
    return mx_planes_bytes(M, N, K, leaf, k_first) + (mx_retiles(M) && K % 128 == 0 ? mxfp8_retiled_scales_bytes(M, N, K) : 0);
}

int tbik_gemm_mxfp8(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                    const void *Ws, int64_t ldws, void *Y, int64_t ldy, tbik_dtype y_dtype, tbik_dtype x_dtype,
                    int M, int N, int K, int leaf, int k_first,
                    void *workspace, size_t workspace_bytes, void *hip_stream) {
    int sl, ns;
    int rc = mxfp8_checks((int)x_dtype, X, ldx, Xs, ldxs, Wt, ldwt, Ws, ldws, M, N, K, leaf, k_first, 1, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (y_dtype != TBIK_F32 && y_dtype != TBIK_BF16) return TBIK_ERR_DTYPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!Y) return TBIK_ERR_NULL;
    if (ldy < N) return TBIK_ERR_SHAPE;
    if (!aligned(Y, y_dtype == TBIK_F32 ? 4 : 2)) return TBIK_ERR_ALIGN;
    const size_t need = tbik_gemm_mxfp8_workspace_bytes(M, N, K, leaf, k_first);
    if (need > 0 && (!workspace || workspace_bytes < need)) return TBIK_ERR_WORKSPACE;
    if (workspace && !aligned(workspace, 256)) return TBIK_ERR_ALIGN;
    hipStream_t s = (hipStream_t)hip_stream;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, nullptr, Y, ldy, (int)y_dtype, M, N, K, sl, ns, 1, (int)x_dtype, 0};
    const Mxfp4Scales sc{(const uint8_t *)Xs, ldxs, (const uint8_t *)Ws, ldws};
    const int split = internal_split(M, N, K, ns);
    const int rows = fp8_tile_rows(M, N);
    GemmArgs probe = a;
    probe.P = split;
    const bool tiled = g_forced_variant.load() != VARIANT_REFERENCE && gemm_mxfp8_tiled_supports(probe, sc);
    hipError_t e;
    void *retiled = (tiled && mx_retiles(M)) ? static_cast<char *>(workspace) + mx_planes_bytes(M, N, K, leaf, k_first) : nullptr;
    if (!tiled) {
        e = launch_gemm_mxfp8_reference(a, sc, s);
    } else if (split == 1) {
        e = launch_gemm_mxfp8_tiled(a, sc, rows, retiled, s);
    } else {
        a.partials = reinterpret_cast<float *>(workspace);
        a.Y = nullptr;
        a.P = split;
        e = launch_gemm_mxfp8_tiled(a, sc, rows, retiled, s);
        if (e == hipSuccess) e = launch_tree_combine(a.partials, split, Y, ldy, (int)y_dtype, M, N, s);
    }
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_gemm_shard_partials_mxfp8(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                                   const void *Ws, int64_t ldws, float *partials, tbik_dtype x_dtype,
                                   int M, int N, int K, int leaf, int k_first, int P,
                                   void *workspace, size_t workspace_bytes, void *hip_stream) {
    int sl, ns;
    int rc = mxfp8_checks((int)x_dtype, X, ldx, Xs, ldxs, Wt, ldwt, Ws, ldws, M, N, K, leaf, k_first, P, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!partials) return TBIK_ERR_NULL;
    if (!aligned(partials, 16)) return TBIK_ERR_ALIGN;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, partials, nullptr, 0, TBIK_F32, M, N, K, sl, ns, P, (int)x_dtype, 0};
    const Mxfp4Scales sc{(const uint8_t *)Xs, ldxs, (const uint8_t *)Ws, ldws};
    const bool tiled = g_forced_variant.load() != VARIANT_REFERENCE && gemm_mxfp8_tiled_supports(a, sc);
    // a workspace as tbik_gemm_mxfp8 takes it has room for the re-tiled scales behind the planes of the K cut
    void *retiled = (tiled && mx_retiles(M) && workspace && aligned(workspace, 256) &&
                     workspace_bytes >= tbik_gemm_mxfp8_workspace_bytes(M, N, K, leaf, k_first))
                        ? static_cast<char *>(workspace) + mx_planes_bytes(M, N, K, leaf, k_first) : nullptr;
    hipError_t e = tiled ? launch_gemm_mxfp8_tiled(a, sc, fp8_tile_rows(M, N), retiled, (hipStream_t)hip_stream)
                         : launch_gemm_mxfp8_reference(a, sc, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_gemm_reference_mxfp8(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                              const void *Ws, int64_t ldws, float *partials, void *Y, int64_t ldy, tbik_dtype y_dtype,
                              tbik_dtype x_dtype, int M, int N, int K, int leaf, int k_first, int P, void *hip_stream) {
    int sl, ns;
    int rc = mxfp8_checks((int)x_dtype, X, ldx, Xs, ldxs, Wt, ldwt, Ws, ldws, M, N, K, leaf, k_first, P, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (y_dtype != TBIK_F32 && y_dtype != TBIK_BF16) return TBIK_ERR_DTYPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!partials && !Y) return TBIK_ERR_NULL;
    if (Y && P != 1) return TBIK_ERR_SHARDS;
    if (Y && ldy < N) return TBIK_ERR_SHAPE;
    if (Y && !aligned(Y, y_dtype == TBIK_F32 ? 4 : 2)) return TBIK_ERR_ALIGN;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, partials, Y, ldy, (int)y_dtype, M, N, K, sl, ns, P, (int)x_dtype, 0};
    const Mxfp4Scales sc{(const uint8_t *)Xs, ldxs, (const uint8_t *)Ws, ldws};
    hipError_t e = launch_gemm_mxfp8_reference(a, sc, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

// ---- MXFP6 operands: one tile shape (128 x 128), so the K cut is that of a 128-row tile whatever M ----
static int mxfp6_split(int M, int N, int ns) {
    const int64_t tiles = (((int64_t)M + 127) / 128) * (((int64_t)N + 127) / 128);
    int split = 1;
    while (ns / split > 16 && split < TBIK_MAX_SHARDS) split *= 2;     // the tiled kernel walks at most 16 superleaves per shard
    if (tiles >= 128) return split;
    while (split < ns && split < 16 && tiles * split < 256) split *= 2;
    return split;
}

static int mxfp6_checks(int x_dtype, const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                        const void *Ws, int64_t ldws, int M, int N, int K, int leaf, int k_first, int P, int *sl, int *ns) {
    int rc = check_tree(M, N, K, leaf, k_first, P, sl, ns);
    if (rc != TBIK_OK) return rc;
    if (x_dtype != TBIK_FP6_E2M3 && x_dtype != TBIK_FP6_E3M2) return TBIK_ERR_DTYPE;
    if (*sl % 64 != 0) return TBIK_ERR_SHAPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!X || !Wt || !Xs || !Ws) return TBIK_ERR_NULL;
    if (ldx < (int64_t)K / 4 * 3 || ldwt < (int64_t)K / 4 * 3 || ldxs < K / 32 || ldws < K / 32) return TBIK_ERR_SHAPE;
    if (!aligned(X, 16) || !aligned(Wt, 16) || ldx % 16 != 0 || ldwt % 16 != 0) return TBIK_ERR_ALIGN;
    return TBIK_OK;
}

size_t tbik_gemm_mxfp6_workspace_bytes(int M, int N, int K, int leaf, int k_first) {
    int sl, ns;
    if (check_tree(M, N, K, leaf, k_first, 1, &sl, &ns) != TBIK_OK) return 0;
    const int split = mxfp6_split(M, N, ns);
    const size_t planes = split > 1 ? (((size_t)split * (size_t)M * (size_t)N * sizeof(float) + 255) & ~(size_t)255) : 0;
    return planes + (mx_retiles(M) && K % 128 == 0 ? mxfp6_retiled_scales_bytes(M, N, K) : 0);
}

int tbik_gemm_mxfp6(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                    const void *Ws, int64_t ldws, void *Y, int64_t ldy, tbik_dtype y_dtype, tbik_dtype x_dtype,
                    int M, int N, int K, int leaf, int k_first,
                    void *workspace, size_t workspace_bytes, void *hip_stream) {
    int sl, ns;
    int rc = mxfp6_checks((int)x_dtype, X, ldx, Xs, ldxs, Wt, ldwt, Ws, ldws, M, N, K, leaf, k_first, 1, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (y_dtype != TBIK_F32 && y_dtype != TBIK_BF16) return TBIK_ERR_DTYPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!Y) return TBIK_ERR_NULL;
    if (ldy < N) return TBIK_ERR_SHAPE;
    if (!aligned(Y, y_dtype == TBIK_F32 ? 4 : 2)) return TBIK_ERR_ALIGN;
    const size_t need = tbik_gemm_mxfp6_workspace_bytes(M, N, K, leaf, k_first);
    if (need > 0 && (!workspace || workspace_bytes < need)) return TBIK_ERR_WORKSPACE;
    if (workspace && !aligned(workspace, 256)) return TBIK_ERR_ALIGN;
    hipStream_t s = (hipStream_t)hip_stream;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, nullptr, Y, ldy, (int)y_dtype, M, N, K, sl, ns, 1, (int)x_dtype, 0};
    const Mxfp4Scales sc{(const uint8_t *)Xs, ldxs, (const uint8_t *)Ws, ldws};
    const int split = mxfp6_split(M, N, ns);
    GemmArgs probe = a;
    probe.P = split;
    const bool tiled = g_forced_variant.load() != VARIANT_REFERENCE && gemm_mxfp6_tiled_supports(probe, sc);
    const size_t planes = split > 1 ? (((size_t)split * (size_t)M * (size_t)N * sizeof(float) + 255) & ~(size_t)255) : 0;
    void *retiled = (tiled && mx_retiles(M)) ? static_cast<char *>(workspace) + planes : nullptr;
    hipError_t e;
    if (!tiled) {
        e = launch_gemm_mxfp6_reference(a, sc, s);
    } else if (split == 1) {
        e = launch_gemm_mxfp6_tiled(a, sc, retiled, s);
    } else {
        a.partials = reinterpret_cast<float *>(workspace);
        a.Y = nullptr;
        a.P = split;
        e = launch_gemm_mxfp6_tiled(a, sc, retiled, s);
        if (e == hipSuccess) e = launch_tree_combine(a.partials, split, Y, ldy, (int)y_dtype, M, N, s);
    }
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_gemm_shard_partials_mxfp6(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                                   const void *Ws, int64_t ldws, float *partials, tbik_dtype x_dtype,
                                   int M, int N, int K, int leaf, int k_first, int P,
                                   void *workspace, size_t workspace_bytes, void *hip_stream) {
    int sl, ns;
    int rc = mxfp6_checks((int)x_dtype, X, ldx, Xs, ldxs, Wt, ldwt, Ws, ldws, M, N, K, leaf, k_first, P, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!partials) return TBIK_ERR_NULL;
    if (!aligned(partials, 16)) return TBIK_ERR_ALIGN;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, partials, nullptr, 0, TBIK_F32, M, N, K, sl, ns, P, (int)x_dtype, 0};
    const Mxfp4Scales sc{(const uint8_t *)Xs, ldxs, (const uint8_t *)Ws, ldws};
    const bool tiled = g_forced_variant.load() != VARIANT_REFERENCE && gemm_mxfp6_tiled_supports(a, sc);
    // a workspace as tbik_gemm_mxfp6 takes it has room for the re-tiled scales behind the planes of the K cut
    const int own_split = mxfp6_split(M, N, ns);
    const size_t planes = own_split > 1 ? (((size_t)own_split * (size_t)M * (size_t)N * sizeof(float) + 255) & ~(size_t)255) : 0;
    void *retiled = (tiled && mx_retiles(M) && workspace && aligned(workspace, 256) &&
                     workspace_bytes >= tbik_gemm_mxfp6_workspace_bytes(M, N, K, leaf, k_first))
                        ? static_cast<char *>(workspace) + planes : nullptr;
    hipError_t e = tiled ? launch_gemm_mxfp6_tiled(a, sc, retiled, (hipStream_t)hip_stream)
                         : launch_gemm_mxfp6_reference(a, sc, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_gemm_reference_mxfp6(const void *X, int64_t ldx, const void *Xs, int64_t ldxs, const void *Wt, int64_t ldwt,
                              const void *Ws, int64_t ldws, float *partials, void *Y, int64_t ldy, tbik_dtype y_dtype,
                              tbik_dtype x_dtype, int M, int N, int K, int leaf, int k_first, int P, void *hip_stream) {
    int sl, ns;
    int rc = mxfp6_checks((int)x_dtype, X, ldx, Xs, ldxs, Wt, ldwt, Ws, ldws, M, N, K, leaf, k_first, P, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (y_dtype != TBIK_F32 && y_dtype != TBIK_BF16) return TBIK_ERR_DTYPE;
    if (M == 0 || N == 0) return TBIK_OK;
    if (!partials && !Y) return TBIK_ERR_NULL;
    if (Y && P != 1) return TBIK_ERR_SHARDS;
    if (Y && ldy < N) return TBIK_ERR_SHAPE;
    if (Y && !aligned(Y, y_dtype == TBIK_F32 ? 4 : 2)) return TBIK_ERR_ALIGN;
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)Wt, ldwt, partials, Y, ldy, (int)y_dtype, M, N, K, sl, ns, P, (int)x_dtype, 0};
    const Mxfp4Scales sc{(const uint8_t *)Xs, ldxs, (const uint8_t *)Ws, ldws};
    hipError_t e = launch_gemm_mxfp6_reference(a, sc, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

// How tbik_gemm_swiglu runs a shape (pure): the K split of the [M, 2 I] GEMM, and whether the unsplit case can end in
// the 128 x 128 tile's activation epilogue or has to pass gate and up through a 16-bit staging buffer.
enum { SWIGLU_FUSED = 0, SWIGLU_SPLIT = 1, SWIGLU_STAGED = 2 };
static int swiglu_route(int dtype, int M, int I, int K, int sl, int ns, int *split) {
    const int N = 2 * I;
    GemmArgs probe{nullptr, K, nullptr, N, nullptr, nullptr, I, dtype, M, N, K, sl, ns, 1, dtype, 0};
    probe.P = *split = internal_split(M, N, K, ns);
    if (*split > 1) return pick_variant(probe) != VARIANT_REFERENCE ? SWIGLU_SPLIT : SWIGLU_STAGED;
    probe.swiglu = 1;
    return (tile_rows(M, N) == 128 && g_forced_variant.load() == VARIANT_AUTO && gemm_tiled_supports(probe, VARIANT_T128))
               ? SWIGLU_FUSED : SWIGLU_STAGED;
}

size_t tbik_gemm_swiglu_workspace_bytes(int M, int I, int K, int leaf, int k_first) {
    int sl, ns, split;
    if (I <= 0 || I > 0x3fffffff || check_tree(M, 2 * I, K, leaf, k_first, 1, &sl, &ns) != TBIK_OK) return 0;
    switch (swiglu_route(TBIK_BF16, M, I, K, sl, ns, &split)) {
        case SWIGLU_FUSED: return 0;
        case SWIGLU_SPLIT: return (size_t)split * (size_t)M * (size_t)(2 * I) * sizeof(float);
        default: return (((size_t)M * (size_t)(2 * I) * 2 + 255) & ~(size_t)255) + tbik_gemm_workspace_bytes(M, 2 * I, K, leaf, k_first);
    }
}

int tbik_silu_mul(const void *gate, int64_t ldg, const void *up, int64_t ldu, void *act, int64_t lda,
                  tbik_dtype dtype, int M, int I, void *hip_stream) {
    if (M < 0 || I < 0) return TBIK_ERR_SHAPE;
    if (dtype != TBIK_BF16 && dtype != TBIK_F16) return TBIK_ERR_DTYPE;
    if (M == 0 || I == 0) return TBIK_OK;
    if (!gate || !up || !act) return TBIK_ERR_NULL;
    if (ldg < I || ldu < I || lda < I) return TBIK_ERR_SHAPE;
    hipError_t e = launch_silu_mul((const uint16_t *)gate, ldg, (const uint16_t *)up, ldu, (uint16_t *)act, lda, (int)dtype, M, I,
                                   (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_gemm_swiglu(const void *X, int64_t ldx, const void *W_gu, int64_t ldw, void *act, int64_t lda,
                     tbik_dtype dtype, int M, int I, int K, int leaf, int k_first,
                     void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (I < 0 || I > 0x3fffffff || I % 8 != 0) return TBIK_ERR_SHAPE;
    const int N = 2 * I;
    int sl, ns;
    int rc = check_tree(M, N, K, leaf, k_first, 1, &sl, &ns);
    if (rc != TBIK_OK) return rc;
    if (dtype != TBIK_BF16 && dtype != TBIK_F16) return TBIK_ERR_DTYPE;
    if (M == 0 || I == 0) return TBIK_OK;
    rc = check_operands((int)dtype, X, ldx, W_gu, ldw, N, K);
    if (rc != TBIK_OK) return rc;
    if (ldx >= (1 << 22) || ldw >= (1 << 22)) return TBIK_ERR_SHAPE;
    if (!act) return TBIK_ERR_NULL;
    if (lda < I) return TBIK_ERR_SHAPE;
    if (!aligned(act, 2)) return TBIK_ERR_ALIGN;
    const size_t need = tbik_gemm_swiglu_workspace_bytes(M, I, K, leaf, k_first);
    if (need > 0 && (!workspace || workspace_bytes < need)) return TBIK_ERR_WORKSPACE;
    if (workspace && !aligned(workspace, 256)) return TBIK_ERR_ALIGN;

    hipStream_t s = (hipStream_t)hip_stream;
    int split;
    const int route = swiglu_route((int)dtype, M, I, K, sl, ns, &split);
    GemmArgs a{(const uint16_t *)X, ldx, (const uint16_t *)W_gu, ldw, nullptr, act, lda, (int)dtype, M, N, K, sl, ns, 1, (int)dtype, 0};
    hipError_t e;
    if (route == SWIGLU_FUSED) {
        a.swiglu = 1;
        e = launch_gemm_tiled(a, VARIANT_T128, s);
    } else if (route == SWIGLU_SPLIT) {
        a.partials = reinterpret_cast<float *>(workspace);
        a.Y = nullptr;
        a.P = split;
        e = launch_tiled(a, pick_variant(a), s);
        if (e == hipSuccess) e = launch_tree_combine_swiglu(a.partials, split, (uint16_t *)act, lda, (int)dtype, M, I, s);
    } else {
        uint16_t *staged = reinterpret_cast<uint16_t *>(workspace);
        const size_t staged_bytes = ((size_t)M * (size_t)N * 2 + 255) & ~(size_t)255;
        rc = gemm((int)dtype, X, ldx, W_gu, ldw, staged, N, (int)dtype, M, N, K, leaf, k_first,
                  reinterpret_cast<char *>(workspace) + staged_bytes, workspace_bytes - staged_bytes, hip_stream);
        if (rc != TBIK_OK) return rc;
        e = launch_silu_mul(staged, N, staged + I, N, (uint16_t *)act, lda, (int)dtype, M, I, s);
    }
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_tree_allreduce(float *bufs, int P, int64_t n, void *hip_stream) {
    if (n < 0) return TBIK_ERR_SHAPE;
    if (P < 1 || !is_pow2(P) || P > TBIK_MAX_SHARDS) return TBIK_ERR_SHARDS;
    if (n == 0) return TBIK_OK;
    if (!bufs) return TBIK_ERR_NULL;
    if (!aligned(bufs, 16)) return TBIK_ERR_ALIGN;
    hipError_t e = launch_tree_allreduce(bufs, P, n, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

static int rmsnorm(int dtype, const void *x, const void *weight, void *y, int M, int H, float eps, void *hip_stream) {
    if (M < 0 || H <= 0 || H % 8 != 0 || H > 65536) return TBIK_ERR_SHAPE;
    if (M == 0) return TBIK_OK;
    if (!x || !weight || !y) return TBIK_ERR_NULL;
    if (!aligned(x, 16) || !aligned(weight, 16) || !aligned(y, 16)) return TBIK_ERR_ALIGN;
    hipError_t e = launch_rmsnorm((const uint16_t *)x, (const uint16_t *)weight, (uint16_t *)y, M, H, eps, dtype,
                                  (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_rmsnorm(const void *x, const void *weight, void *y, int M, int H, float eps, void *hip_stream) {
    return rmsnorm(TBIK_BF16, x, weight, y, M, H, eps, hip_stream);
}

int tbik_rmsnorm_f16(const void *x, const void *weight, void *y, int M, int H, float eps, void *hip_stream) {
    return rmsnorm(TBIK_F16, x, weight, y, M, H, eps, hip_stream);
}

static int attention(int dtype, const void *Q, const void *K, const void *V, void *O,
                     const int32_t *cu_seqlens_q, const int32_t *cu_seqlens_k, int batch, int max_seqlen_q, int max_seqlen_k,
                     int total_q, int total_k, int heads_q, int heads_kv, int head_dim,
                     int64_t q_stride, int64_t k_stride, int64_t v_stride, int64_t o_stride,
                     float scale, int causal, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (batch < 0 || max_seqlen_q < 0 || max_seqlen_k < 0 || total_q < 0 || total_k < 0 || heads_q <= 0 || heads_kv <= 0 ||
        head_dim <= 0)
        return TBIK_ERR_SHAPE;
    if (heads_q % heads_kv != 0 || heads_q > 65535 || batch > 65535) return TBIK_ERR_SHAPE;
    if (head_dim != 128) return TBIK_ERR_UNSUPPORTED;
    if (q_stride >= (1 << 24) || k_stride >= (1 << 24) || v_stride >= (1 << 24) || o_stride >= (1 << 24)) return TBIK_ERR_SHAPE;
    if (q_stride < (int64_t)heads_q * head_dim || o_stride < (int64_t)heads_q * head_dim ||
        k_stride < (int64_t)heads_kv * head_dim || v_stride < (int64_t)heads_kv * head_dim)
        return TBIK_ERR_SHAPE;
    if (batch == 0 || max_seqlen_q == 0 || total_q == 0) return TBIK_OK;
    if (!Q || !O || !cu_seqlens_q || !cu_seqlens_k) return TBIK_ERR_NULL;
    if (total_k > 0 && (!K || !V)) return TBIK_ERR_NULL;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) || !aligned(cu_seqlens_q, 4) ||
        !aligned(cu_seqlens_k, 4) || q_stride % 8 || k_stride % 8 || v_stride % 8 || o_stride % 8)
        return TBIK_ERR_ALIGN;
    if (max_seqlen_k > total_k) max_seqlen_k = total_k;          // no sequence has more keys than the call
    const size_t need = attention_workspace(batch, max_seqlen_q, max_seqlen_k, heads_q, heads_kv);
    if (need > 0 && (!workspace || workspace_bytes < need)) return TBIK_ERR_WORKSPACE;
    if (need > 0 && !aligned(workspace, 256)) return TBIK_ERR_ALIGN;
    AttnArgs a{(const uint16_t *)Q, (const uint16_t *)K, (const uint16_t *)V, (uint16_t *)O, dtype, cu_seqlens_q, cu_seqlens_k,
               batch, max_seqlen_q, max_seqlen_k, total_q, total_k, heads_q, heads_kv, q_stride, k_stride, v_stride, o_stride,
               scale, causal != 0, need > 0 ? workspace : nullptr, need > 0 ? workspace_bytes : 0};
    hipError_t e = launch_attention(a, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_attention(const void *Q, const void *K, const void *V, void *O,
                   const int32_t *cu_seqlens_q, const int32_t *cu_seqlens_k, int batch, int max_seqlen_q, int max_seqlen_k,
                   int total_q, int total_k, int heads_q, int heads_kv, int head_dim,
                   int64_t q_stride, int64_t k_stride, int64_t v_stride, int64_t o_stride,
                   float scale, int causal, void *workspace, size_t workspace_bytes, void *hip_stream) {
    return attention(TBIK_BF16, Q, K, V, O, cu_seqlens_q, cu_seqlens_k, batch, max_seqlen_q, max_seqlen_k, total_q, total_k, heads_q,
                     heads_kv, head_dim, q_stride, k_stride, v_stride, o_stride, scale, causal, workspace, workspace_bytes,
                     hip_stream);
}

int tbik_attention_f16(const void *Q, const void *K, const void *V, void *O,
                       const int32_t *cu_seqlens_q, const int32_t *cu_seqlens_k, int batch, int max_seqlen_q, int max_seqlen_k,
                       int total_q, int total_k, int heads_q, int heads_kv, int head_dim,
                       int64_t q_stride, int64_t k_stride, int64_t v_stride, int64_t o_stride,
                       float scale, int causal, void *workspace, size_t workspace_bytes, void *hip_stream) {
    return attention(TBIK_F16, Q, K, V, O, cu_seqlens_q, cu_seqlens_k, batch, max_seqlen_q, max_seqlen_k, total_q, total_k, heads_q,
                     heads_kv, head_dim, q_stride, k_stride, v_stride, o_stride, scale, causal, workspace, workspace_bytes,
                     hip_stream);
}

size_t tbik_attention_workspace_bytes(int batch, int max_seqlen_q, int max_seqlen_k, int heads_q, int heads_kv) {
    return attention_workspace(batch, max_seqlen_q, max_seqlen_k, heads_q, heads_kv);
}

int tbik_set_attention_variant(int variant) { return set_attention_variant(variant) < 0 ? TBIK_ERR_DTYPE : TBIK_OK; }

size_t tbik_row_reduce_workspace_bytes(int M, int64_t V, tbik_rowop op) {
    if (op != TBIK_SUM && op != TBIK_MAX && op != TBIK_LOGSOFTMAX) return 0;
    // sized for the finer of the two input types (fp32 rows have twice the leaves of 16-bit rows)
    return row_reduce_workspace(M, V, TBIK_F32, (int)op);
}

static int combine_residual_rmsnorm(int dtype, const float *partials, int P, const void *residual, const void *weight,
                                    float eps, void *hidden, void *normed, int M, int H, void *hip_stream) {
    if (M < 0 || H <= 0 || H % 8 != 0 || H > 65536) return TBIK_ERR_SHAPE;
    if (P < 1 || !is_pow2(P) || P > TBIK_MAX_SHARDS) return TBIK_ERR_SHARDS;
    if (P > 16) return TBIK_ERR_UNSUPPORTED;
    if (M == 0) return TBIK_OK;
    if (!partials || !residual || !weight || !hidden || !normed) return TBIK_ERR_NULL;
    if (!aligned(partials, 16) || !aligned(residual, 16) || !aligned(weight, 16) || !aligned(hidden, 16) || !aligned(normed, 16))
        return TBIK_ERR_ALIGN;
    if (normed == hidden || normed == residual) return TBIK_ERR_SHAPE;      // only hidden may share residual's buffer
    hipError_t e = launch_combine_residual_rmsnorm(partials, P, (const uint16_t *)residual, (const uint16_t *)weight,
                                                   (uint16_t *)hidden, (uint16_t *)normed, M, H, eps, dtype,
                                                   (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_combine_residual_rmsnorm(const float *partials, int P, const void *residual, const void *weight, float eps,
                                  void *hidden, void *normed, int M, int H, void *hip_stream) {
    return combine_residual_rmsnorm(TBIK_BF16, partials, P, residual, weight, eps, hidden, normed, M, H, hip_stream);
}

int tbik_combine_residual_rmsnorm_f16(const float *partials, int P, const void *residual, const void *weight, float eps,
                                      void *hidden, void *normed, int M, int H, void *hip_stream) {
    return combine_residual_rmsnorm(TBIK_F16, partials, P, residual, weight, eps, hidden, normed, M, H, hip_stream);
}

int tbik_row_reduce(const void *x, tbik_dtype x_dtype, void *out, tbik_rowop op, int M, int64_t V,
                    void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (x_dtype != TBIK_F32 && x_dtype != TBIK_BF16 && x_dtype != TBIK_F16) return TBIK_ERR_DTYPE;
    if (op != TBIK_SUM && op != TBIK_MAX && op != TBIK_LOGSOFTMAX) return TBIK_ERR_DTYPE;
    const int epl = (x_dtype == TBIK_F32) ? 4 : 8;
    if (M < 0 || V <= 0 || V % epl != 0) return TBIK_ERR_SHAPE;
    if (M == 0) return TBIK_OK;
    if (!x || !out) return TBIK_ERR_NULL;
    if (!aligned(x, 16) || !aligned(out, op == TBIK_LOGSOFTMAX ? 16 : 4)) return TBIK_ERR_ALIGN;
    const size_t need = row_reduce_workspace(M, V, (int)x_dtype, (int)op);
    if (!workspace || workspace_bytes < need) return TBIK_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return TBIK_ERR_ALIGN;
    hipError_t e = launch_row_reduce(x, (int)x_dtype, out, (int)op, M, V, workspace, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_row_reduce_static(const void *x, tbik_dtype x_dtype, void *out, tbik_rowop op, int M, int64_t V, void *hip_stream) {
    if (x_dtype != TBIK_F32 && x_dtype != TBIK_BF16 && x_dtype != TBIK_F16) return TBIK_ERR_DTYPE;
    if (op != TBIK_SUM && op != TBIK_MAX && op != TBIK_LOGSOFTMAX) return TBIK_ERR_DTYPE;
    const int epl = (x_dtype == TBIK_F32) ? 4 : 8;
    if (M < 0 || V <= 0 || V % epl != 0) return TBIK_ERR_SHAPE;
    if (M > 0) {
        if (!x || !out) return TBIK_ERR_NULL;
        if (!aligned(x, 16) || !aligned(out, op == TBIK_LOGSOFTMAX ? 16 : 4)) return TBIK_ERR_ALIGN;
        if (row_reduce_workspace(M, V, (int)x_dtype, (int)op) > (size_t)TBIK_STATIC_SCRATCH_BYTES) return TBIK_ERR_WORKSPACE;
    }
    hipError_t e = launch_row_reduce_static(x, (int)x_dtype, out, (int)op, M, V, (hipStream_t)hip_stream);
    return e == hipSuccess ? TBIK_OK : hip_fail(e);
}

int tbik_set_row_wait_limit(int polls) { return set_row_wait_limit(polls); }

int tbik_set_gemm_variant(int variant) {
    if (variant < 0 || variant >= VARIANT_COUNT) return TBIK_ERR_UNSUPPORTED;
    g_forced_variant.store(variant);
    return TBIK_OK;
}

const char *tbik_variant_name(int variant) {
    return (variant >= 0 && variant < VARIANT_COUNT) ? kVariantNames[variant] : nullptr;
}

const char *tbik_status_string(int status) {
    switch (status) {
        case TBIK_OK: return "ok";
        case TBIK_ERR_NULL: return "null pointer";
        case TBIK_ERR_SHAPE: return "illegal shape or tree parameters";
        case TBIK_ERR_SHARDS: return "illegal shard count";
        case TBIK_ERR_DTYPE: return "illegal dtype or op";
        case TBIK_ERR_ALIGN: return "misaligned pointer or leading dimension";
        case TBIK_ERR_WORKSPACE: return "workspace missing or too small";
        case TBIK_ERR_UNSUPPORTED: return "unsupported";
        case TBIK_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int tbik_last_hip_error(void) { return g_last_hip_error.load(); }

const char *tbik_version(void) { return "tbik-gfx950 0.1"; }

}  // extern "C"
