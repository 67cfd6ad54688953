// Host side of the C ABI declared in include/flexq.h: argument validation,
// the layer / plan handles and the launches.  Validation happens before any
// HIP call so every error path can be exercised on a host without a GPU.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstddef>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/flexq.h"
#include "fq_internal.h"

namespace {

thread_local char g_err[256] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char *what)
{
    return fail(FQ_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

constexpr uint32_t LAYER_MAGIC = 0x46514C59u; // "FQLY"
constexpr uint32_t PLAN_MAGIC = 0x4651504Cu;  // "FQPL"
// The batch-1 decode kernel keeps one row of x (plus its slice sums) in LDS: 72 KiB at this K, two
// workgroups per CU.  The widest row of the models the paper runs is 28672 (Llama-70B's FFN).
constexpr int MAX_DECODE_K = FQ_MAX_DECODE_K;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int slot_of(int bits) { return bits == 4 ? 0 : bits == 8 ? 1 : bits == 16 ? 2 : bits == 2 ? 3 : bits == 3 ? 4 : -1; }

} // namespace

struct fq_layer {
    uint32_t magic;
    int N, K, group;
    const void *codes[5]; // by slot_of(bits)
    const void *scales[5];
    const void *zeros[5];
};

struct fq_plan {
    uint32_t magic;
    FqPlanGeom geom;
    // stage-ordered plans (fq_plan_create_staged): n_stages > 0
    int n_stages;
    const int32_t *stage_begin_dev; // int32 [n_stages + 1], after the table
    int *sync_dev;                  // the barrier's counters and the status words, after that
    long long wait_limit;           // polls a workgroup spends on one stage boundary before it gives up
    const FqLinearDesc *table_dev;
    int *queue_dev;  // after the table: per-XCD tile cursors, a count of finished workgroups, list totals
    void *order_dev; // after the queue: a list of two ints per entry
};

namespace {

int check_layer(const fq_layer *l)
{
    if (!l)
        return fail(FQ_ERR_NULL, "layer is NULL");
    if (l->magic != LAYER_MAGIC)
        return fail(FQ_ERR_NULL, "layer handle is not valid (destroyed or corrupted)");
    return FQ_OK;
}

void fill_desc(FqLinearDesc &d, const fq_layer *l, const void *x, void *y)
{
    memset(&d, 0, sizeof d);
    d.codes4 = (const uint8_t *)l->codes[0];
    d.scales4 = (const float *)l->scales[0];
    d.zeros4 = (const uint8_t *)l->zeros[0];
    d.codes8 = (const uint8_t *)l->codes[1];
    d.scales8 = (const float *)l->scales[1];
    d.zeros8 = (const uint8_t *)l->zeros[1];
    d.w16 = (const uint16_t *)l->codes[2];
    d.codes2 = (const uint8_t *)l->codes[3];
    d.scales2 = (const float *)l->scales[3];
    d.zeros2 = (const uint8_t *)l->zeros[3];
    d.codes3 = (const uint8_t *)l->codes[4];
    d.scales3 = (const float *)l->scales[4];
    d.zeros3 = (const uint8_t *)l->zeros[4];
    d.x = (const uint16_t *)x;
    d.y = (uint16_t *)y;
    d.N = l->N;
    d.K = l->K;
}

// per_row: group = K (one scale per weight row: 8-bit copies for fq_linear_w8a8) is accepted as well
int check_shape(int N, int K, int group, bool per_row = false)
{
    if (N < 1 || K < 1)
        return fail(FQ_ERR_SHAPE, "N and K must be >= 1 (got N=%d K=%d)", N, K);
    if (per_row && group == K && group != FQ_GROUP) {
        if (K % FQ_GROUP != 0 || K > FQ_MAX_ROW_GROUP_K)
            return fail(FQ_ERR_SHAPE, "group = K needs K a multiple of %d and at most %d (got %d)", FQ_GROUP,
                        FQ_MAX_ROW_GROUP_K, K);
        return FQ_OK;
    }
    if (group != FQ_GROUP)
        return fail(FQ_ERR_SHAPE, "group must be %d%s (got %d)", FQ_GROUP, per_row ? " or K" : "", group);
    if (K % group != 0)
        return fail(FQ_ERR_SHAPE, "K=%d is not a multiple of group=%d", K, group);
    return FQ_OK;
}

// A layer whose copies are quantized per row is served by fq_linear_w8a8 only.
int check_group128(const fq_layer *l, const char *who)
{
    if (l->group != FQ_GROUP)
        return fail(FQ_ERR_SHAPE, "%s: the layer's copies have one scale per row (group = K = %d): they are served by "
                                  "fq_linear_w8a8 only", who, l->K);
    return FQ_OK;
}

} // namespace

extern "C" {

const char *fq_last_error(void) { return g_err; }

int fq_packed_sizes(int N, int K, int bits, int group, size_t *codes_bytes, size_t *scales_bytes,
                    size_t *zeros_bytes)
{
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8)
        return fail(FQ_ERR_BITS, "fq_packed_sizes: bits must be 2, 3, 4 or 8 (got %d)", bits);
    if (int rc = check_shape(N, K, group, bits == 8))
        return rc;
    const size_t groups = (size_t)N * (size_t)(K / group);
    if (codes_bytes)
        *codes_bytes = (size_t)N * (size_t)K * (size_t)bits / 8;
    if (scales_bytes)
        *scales_bytes = groups * sizeof(float);
    if (zeros_bytes)
        *zeros_bytes = groups;
    return FQ_OK;
}

static int quantize_any(const char *who, bool symmetric, const void *w_fp16, int N, int K, int bits, int group,
                        void *codes, void *scales, void *zeros, void *stream)
{
    if (!w_fp16 || !codes || !scales || !zeros)
        return fail(FQ_ERR_NULL, "%s: NULL tensor pointer", who);
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8)
        return fail(FQ_ERR_BITS, "%s: bits must be 2, 3, 4 or 8 (got %d)", who, bits);
    if (int rc = check_shape(N, K, group, bits == 8))
        return rc;
    if (!aligned16(w_fp16) || !aligned16(codes) || (reinterpret_cast<uintptr_t>(scales) & 3u))
        return fail(FQ_ERR_ALIGN, "%s: w and codes need 16-byte, scales 4-byte alignment", who);
    const long long n_groups = (long long)N * (K / group);
    hipError_t e = group != FQ_GROUP
        ? fq_launch_quantize_row8(w_fp16, N, K, symmetric, codes, scales, zeros, (hipStream_t)stream)
        : fq_launch_quantize(w_fp16, n_groups, bits, symmetric, codes, scales, zeros, (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "quantize launch");
    return FQ_OK;
}

int fq_quantize(const void *w_fp16, int N, int K, int bits, int group, void *codes, void *scales,
                void *zeros, void *stream)
{
    return quantize_any("fq_quantize", false, w_fp16, N, K, bits, group, codes, scales, zeros, stream);
}

int fq_quantize_sym(const void *w_fp16, int N, int K, int bits, int group, void *codes, void *scales,
                    void *zeros, void *stream)
{
    return quantize_any("fq_quantize_sym", true, w_fp16, N, K, bits, group, codes, scales, zeros, stream);
}

int fq_fake_quantize(const void *w_fp16, int N, int K, int bits, int group, int symmetric, void *w_hat_fp16,
                     void *stream)
{
    if (!w_fp16 || !w_hat_fp16)
        return fail(FQ_ERR_NULL, "fq_fake_quantize: NULL tensor pointer");
    if (bits < 2 || bits > 8)
        return fail(FQ_ERR_BITS, "fq_fake_quantize: bits must be 2..8 (got %d)", bits);
    if (int rc = check_shape(N, K, group))
        return rc;
    if (!aligned16(w_fp16) || !aligned16(w_hat_fp16))
        return fail(FQ_ERR_ALIGN, "fq_fake_quantize: w and w_hat need 16-byte alignment");
    const long long n_groups = (long long)N * (K / group);
    hipError_t e = fq_launch_fake_quantize(w_fp16, n_groups, bits, symmetric != 0, w_hat_fp16, (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_fake_quantize launch");
    return FQ_OK;
}

int fq_lm_head_entropy(const void *x_fp16, const void *w_fp16, int M, int V, int K, float *logits, float *H,
                       int32_t *argmax, void *stream)
{
    if (M < 1 || M > FQ_MAX_LM_HEAD_M)
        return fail(FQ_ERR_SHAPE, "fq_lm_head_entropy: M must be 1..%d (got %d)", FQ_MAX_LM_HEAD_M, M);
    if (V < 1 || K < 512 || K % 512 != 0 || (long long)M * K > 32768)
        return fail(FQ_ERR_SHAPE,
                    "fq_lm_head_entropy: need V >= 1, K a positive multiple of 512 and M * K <= 32768 (got V=%d K=%d M=%d)",
                    V, K, M);
    if (!x_fp16 || !w_fp16 || !H)
        return fail(FQ_ERR_NULL, "fq_lm_head_entropy: NULL argument");
    if (!aligned16(x_fp16) || !aligned16(w_fp16) || (reinterpret_cast<uintptr_t>(H) & 3u) ||
        (reinterpret_cast<uintptr_t>(logits) & 3u) || (reinterpret_cast<uintptr_t>(argmax) & 3u))
        return fail(FQ_ERR_ALIGN, "fq_lm_head_entropy: x and w need 16-byte, the outputs 4-byte alignment");
    hipError_t e = fq_launch_lm_head_entropy(x_fp16, w_fp16, M, V, K, logits, H, argmax, (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_lm_head_entropy launch");
    return FQ_OK;
}

int fq_layer_create(fq_layer **out, int N, int K, int group)
{
    if (!out)
        return fail(FQ_ERR_NULL, "fq_layer_create: out is NULL");
    *out = nullptr;
    if (int rc = check_shape(N, K, group, true))
        return rc;
    fq_layer *l = new (std::nothrow) fq_layer();
    if (!l)
        return fail(FQ_ERR_HIP, "fq_layer_create: out of host memory");
    l->magic = LAYER_MAGIC;
    l->N = N;
    l->K = K;
    l->group = group;
    *out = l;
    return FQ_OK;
}

int fq_layer_attach(fq_layer *layer, int bits, const void *codes, const void *scales,
                    const void *zeros)
{
    if (int rc = check_layer(layer))
        return rc;
    const int slot = slot_of(bits);
    if (slot < 0)
        return fail(FQ_ERR_BITS, "fq_layer_attach: bits must be 2, 3, 4, 8 or 16 (got %d)", bits);
    if (layer->group != FQ_GROUP && bits != 8)
        return fail(FQ_ERR_BITS, "fq_layer_attach: a layer with one scale per row (group = K) holds an 8-bit copy only "
                                 "(got %d)", bits);
    if (!codes)
        return fail(FQ_ERR_NULL, "fq_layer_attach: codes is NULL");
    if (bits != 16 && (!scales || !zeros))
        return fail(FQ_ERR_NULL, "fq_layer_attach: scales/zeros are NULL for bits=%d", bits);
    if (!aligned16(codes) || (bits != 16 && (reinterpret_cast<uintptr_t>(scales) & 3u)))
        return fail(FQ_ERR_ALIGN, "fq_layer_attach: codes need 16-byte, scales 4-byte alignment");
    layer->codes[slot] = codes;
    layer->scales[slot] = bits == 16 ? nullptr : scales;
    layer->zeros[slot] = bits == 16 ? nullptr : zeros;
    return FQ_OK;
}

int fq_layer_destroy(fq_layer *layer)
{
    if (int rc = check_layer(layer))
        return rc;
    layer->magic = 0;
    delete layer;
    return FQ_OK;
}

int fq_linear(const fq_layer *layer, int bits, const void *x_fp16, int M, void *y_fp16, void *stream)
{
    if (int rc = check_layer(layer))
        return rc;
    if (int rc = check_group128(layer, "fq_linear"))
        return rc;
    if (!x_fp16 || !y_fp16)
        return fail(FQ_ERR_NULL, "fq_linear: x or y is NULL");
    const int slot = slot_of(bits);
    if (slot < 0)
        return fail(FQ_ERR_BITS, "fq_linear: bits must be 2, 3, 4, 8 or 16 (got %d)", bits);
    if (!layer->codes[slot])
        return fail(FQ_ERR_NOT_ATTACHED, "fq_linear: no %d-bit copy attached to this layer", bits);
    if (M < 1)
        return fail(FQ_ERR_SHAPE, "fq_linear: M must be >= 1 (got %d)", M);
    if (!aligned16(x_fp16) || (reinterpret_cast<uintptr_t>(y_fp16) & 1u))
        return fail(FQ_ERR_ALIGN, "fq_linear: x needs 16-byte and y 2-byte alignment");
    FqLinearDesc d;
    fill_desc(d, layer, x_fp16, y_fp16);
    hipError_t e = hipSuccess;
    if (bits == 3 && (M > FQ_MAX_DECODE_M || layer->K > MAX_DECODE_K)) {
        // The GEMM has no 3-bit unpacking: the small-batch kernel runs the call in slabs of
        // FQ_MAX_DECODE_M batch rows (it walks K in chunks, whatever its length), reading the
        // weights once per slab.
        const int rows = 128;
        const int tiles = (layer->N + rows - 1) / rows;
        for (int m0 = 0; m0 < M && e == hipSuccess; m0 += FQ_MAX_DECODE_M) {
            const int m = M - m0 < FQ_MAX_DECODE_M ? M - m0 : FQ_MAX_DECODE_M;
            d.x = (const uint16_t *)x_fp16 + (size_t)m0 * layer->K;
            d.y = (uint16_t *)y_fp16 + (size_t)m0 * layer->N;
            e = fq_launch_skinny(&d, bits, nullptr, nullptr, 1, tiles, rows, m, true, nullptr, nullptr, (hipStream_t)stream);
        }
    } else if (M <= FQ_MAX_DECODE_M && layer->K <= MAX_DECODE_K) {
        int rows = M == 1 ? fq_decode_tile_rows(layer->N, layer->K, M) : fq_skinny_tile_rows(layer->N, M);
        if (M > 1 && bits == 2 && rows == 16) // the K-split kernel takes 3, 4, 8 and 16 bits
            rows = 64;
        const int tiles = (layer->N + rows - 1) / rows;
        e = M == 1 ? fq_launch_decode(&d, bits, nullptr, nullptr, 1, tiles, rows, layer->K, M, nullptr, (hipStream_t)stream)
                   : fq_launch_skinny(&d, bits, nullptr, nullptr, 1, tiles, rows, M, bits == 3, nullptr, nullptr, (hipStream_t)stream);
    } else {
        e = fq_launch_prefill(d, bits, M, (hipStream_t)stream);
    }
    if (e != hipSuccess)
        return hip_fail(e, "fq_linear launch");
    return FQ_OK;
}

int fq_quantize_act(const void *x_fp16, int M, int K, void *xq, float *sx, int32_t *xsum, void *stream)
{
    if (M < 0 || K < FQ_GROUP || K % FQ_GROUP != 0)
        return fail(FQ_ERR_SHAPE, "fq_quantize_act: need M >= 0 and K a positive multiple of %d (got M=%d K=%d)",
                    FQ_GROUP, M, K);
    if (!x_fp16 || !xq || !sx || !xsum)
        return fail(FQ_ERR_NULL, "fq_quantize_act: NULL argument");
    if (!aligned16(x_fp16) || !aligned16(xq) || (reinterpret_cast<uintptr_t>(sx) & 3u) ||
        (reinterpret_cast<uintptr_t>(xsum) & 3u))
        return fail(FQ_ERR_ALIGN, "fq_quantize_act: x and xq need 16-byte, sx and xsum 4-byte alignment");
    hipError_t e = fq_launch_quantize_act(x_fp16, M, K, xq, sx, xsum, (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_quantize_act launch");
    return FQ_OK;
}

int fq_linear_w8a8(const fq_layer *layer, const void *xq, const float *sx, const int32_t *xsum, int M,
                   void *y_fp16, void *stream)
{
    if (int rc = check_layer(layer))
        return rc;
    if (!xq || !sx || !xsum || !y_fp16)
        return fail(FQ_ERR_NULL, "fq_linear_w8a8: NULL argument");
    if (!layer->codes[slot_of(8)])
        return fail(FQ_ERR_NOT_ATTACHED, "fq_linear_w8a8: no 8-bit copy attached to this layer");
    if (M < 1)
        return fail(FQ_ERR_SHAPE, "fq_linear_w8a8: M must be >= 1 (got %d)", M);
    if (!aligned16(xq) || (reinterpret_cast<uintptr_t>(sx) & 3u) || (reinterpret_cast<uintptr_t>(xsum) & 3u) ||
        (reinterpret_cast<uintptr_t>(y_fp16) & 1u))
        return fail(FQ_ERR_ALIGN, "fq_linear_w8a8: xq needs 16-byte, sx and xsum 4-byte, y 2-byte alignment");
    FqLinearDesc d;
    fill_desc(d, layer, nullptr, y_fp16);
    hipError_t e = fq_launch_w8a8(d, xq, sx, xsum, M, layer->group != FQ_GROUP, (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_linear_w8a8 launch");
    return FQ_OK;
}

size_t fq_plan_workspace_bytes(int count)
{
    if (count < 1)
        return 0;
    // the descriptor table, then 256 bytes for the tile queue of the streaming batch kernel and a
    // list of 8 bytes per entry: what a launch runs under its bit-widths
    return ((size_t)count * sizeof(FqLinearDesc) + 255) / 256 * 256 + 256 + ((size_t)count * 8 + 255) / 256 * 256;
}

} // extern "C"

int fq_fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

// Checks the arguments of a plan (every check that needs no HIP call first, then the device facts
// that size the tiles) and writes its descriptor table and geometry.
int fq_plan_layout(const char *who, int count, const fq_layer *const *layers, const void *const *xs,
                   void *const *ys, int M, FqLinearDesc *table, FqPlanGeom *geom)
{
    if (!layers || !xs || !ys)
        return fail(FQ_ERR_NULL, "%s: NULL argument", who);
    if (count < 1)
        return fail(FQ_ERR_SHAPE, "%s: count must be >= 1 (got %d)", who, count);
    if (M < 1 || M > FQ_MAX_DECODE_M)
        return fail(FQ_ERR_SHAPE, "%s: M must be in 1..%d (got %d)", who, FQ_MAX_DECODE_M, M);
    long long total_rows = 0;
    int max_K = 0;
    bool has2 = false, has3 = false;
    for (int i = 0; i < count; i++) {
        if (int rc = check_layer(layers[i]))
            return rc;
        if (int rc = check_group128(layers[i], who))
            return rc;
        if (!xs[i] || !ys[i])
            return fail(FQ_ERR_NULL, "%s: x or y of entry %d is NULL", who, i);
        if (!aligned16(xs[i]) || (reinterpret_cast<uintptr_t>(ys[i]) & 1u))
            return fail(FQ_ERR_ALIGN, "%s: entry %d: x needs 16-byte, y 2-byte alignment", who, i);
        if (layers[i]->K > MAX_DECODE_K)
            return fail(FQ_ERR_SHAPE, "%s: entry %d: K=%d exceeds the decode limit %d", who, i, layers[i]->K,
                        MAX_DECODE_K);
        if (!layers[i]->codes[0] && !layers[i]->codes[1] && !layers[i]->codes[2] && !layers[i]->codes[3] &&
            !layers[i]->codes[4])
            return fail(FQ_ERR_NOT_ATTACHED, "%s: entry %d has no copy attached", who, i);
        total_rows += layers[i]->N;
        if (layers[i]->K > max_K)
            max_K = layers[i]->K;
        has2 = has2 || layers[i]->codes[3] != nullptr;
        has3 = has3 || layers[i]->codes[4] != nullptr;
    }
    int rows = M == 1 ? fq_decode_tile_rows(total_rows, max_K, M) : fq_skinny_tile_rows(total_rows, M);
    // 256-row tiles at M > 1 mean the streaming kernel, whose tile queue deals runs of 8 tiles to 8
    // XCDs of 8 x k compute units: a device of another shape stays with the register-fed kernel
    if (M > 1 && rows == 256 && fq_device_cus() % 64 != 0)
        rows = 128;
    if (M > 1 && has2 && rows == 16) // the K-split kernel for launches with few rows has no 2-bit path
        rows = 64;
    // the streaming kernel's stages are whole 128-byte lines of a row, which blocks of 12 bytes do not
    // fill evenly: a batched plan that holds a 3-bit copy, whose entries may be switched to it at any
    // token, runs on the register-fed kernel
    if (M > 1 && has3 && rows == 256)
        rows = 128;
    long long tiles = 0;
    for (int i = 0; i < count; i++) {
        fill_desc(table[i], layers[i], xs[i], ys[i]);
        table[i].tile_begin = (int)tiles;
        tiles += (layers[i]->N + rows - 1) / rows;
        if (tiles > 0x7fffffffLL)
            return fail(FQ_ERR_SHAPE, "%s: too many row tiles", who);
    }
    geom->count = count;
    geom->M = M;
    geom->total_tiles = (int)tiles;
    geom->max_K = max_K;
    geom->tile_rows = rows;
    geom->has3 = has3 ? 1 : 0;
    return FQ_OK;
}

static_assert(FQ_BANKS == FQ_SCRATCH_BANKS, "the public header states the number of scratch banks");

hipError_t fq_plan_launch(const FqPlanGeom &g, const FqLinearDesc *table_dev, int *queue_dev, void *order_dev,
                          const int32_t *bits_dev, hipStream_t stream)
{
    hipError_t e = g.M == 1
        ? fq_launch_decode(nullptr, 0, table_dev, bits_dev, g.count, g.total_tiles, g.tile_rows, g.max_K, g.M,
                           queue_dev ? queue_dev + FQ_Q_FLAGS : nullptr, stream)
        : fq_launch_skinny(nullptr, 0, table_dev, bits_dev, g.count, g.total_tiles, g.tile_rows, g.M, g.has3 != 0, queue_dev,
                           order_dev, stream);
    return e;
}

extern "C" {

int fq_plan_create(fq_plan **out, int count, const fq_layer *const *layers, const void *const *xs,
                   void *const *ys, int M, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!out)
        return fail(FQ_ERR_NULL, "fq_plan_create: out is NULL");
    *out = nullptr;
    if (!layers || !xs || !ys || !workspace)
        return fail(FQ_ERR_NULL, "fq_plan_create: NULL argument");
    if (count < 1)
        return fail(FQ_ERR_SHAPE, "fq_plan_create: count must be >= 1 (got %d)", count);
    if (workspace_bytes < fq_plan_workspace_bytes(count))
        return fail(FQ_ERR_SHAPE, "fq_plan_create: workspace too small (%zu < %zu bytes)",
                    workspace_bytes, fq_plan_workspace_bytes(count));
    if (reinterpret_cast<uintptr_t>(workspace) & 255u)
        return fail(FQ_ERR_ALIGN, "fq_plan_create: workspace must be 256-byte aligned");
    std::vector<FqLinearDesc> table((size_t)count);
    FqPlanGeom geom;
    if (int rc = fq_plan_layout("fq_plan_create", count, layers, xs, ys, M, table.data(), &geom))
        return rc;
    fq_plan *p = new (std::nothrow) fq_plan();
    if (!p)
        return fail(FQ_ERR_HIP, "fq_plan_create: out of host memory");
    // The table is small; a synchronous-with-respect-to-host copy keeps the host vector's
    // lifetime trivial (hipMemcpyAsync from pageable memory returns after staging the source).
    const size_t table_bytes = ((size_t)count * sizeof(FqLinearDesc) + 255) / 256 * 256;
    hipError_t e = hipMemcpyAsync(workspace, table.data(), (size_t)count * sizeof(FqLinearDesc),
                                  hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e == hipSuccess) // the queue starts at zero; the kernel that uses it leaves it at zero
        e = hipMemsetAsync((char *)workspace + table_bytes, 0, 256, (hipStream_t)stream);
    if (e == hipSuccess)
        e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) {
        delete p;
        return hip_fail(e, "fq_plan_create table copy");
    }
    p->magic = PLAN_MAGIC;
    p->geom = geom;
    p->table_dev = (const FqLinearDesc *)workspace;
    p->queue_dev = (int *)((char *)workspace + table_bytes);
    p->order_dev = (char *)workspace + table_bytes + 256;
    *out = p;
    return FQ_OK;
}

// Layout of a stage-ordered plan's workspace: table | stage_begin | sync words.
static size_t staged_table_bytes(int count) { return ((size_t)count * sizeof(FqLinearDesc) + 255) / 256 * 256; }
static size_t staged_begin_bytes(int n_stages) { return ((size_t)(n_stages + 1) * 4 + 255) / 256 * 256; }
constexpr size_t STAGED_SYNC_BYTES = FQ_STAGED_SYNC_BYTES;
constexpr int STAGED_RES_CHUNKS = 1024; // 4-row chunks of one stage a workgroup can hold results for
constexpr long long STAGED_WAIT_LIMIT = 1LL << 21; // about a second of polling

size_t fq_plan_staged_workspace_bytes(int count, int n_stages)
{
    if (count < 1 || n_stages < 1 || n_stages > count)
        return 0;
    return staged_table_bytes(count) + staged_begin_bytes(n_stages) + STAGED_SYNC_BYTES;
}

int fq_plan_create_staged(fq_plan **out, int count, const fq_layer *const *layers, const void *const *xs,
                          void *const *ys, const int32_t *stage, int M, void *workspace, size_t workspace_bytes,
                          void *stream)
{
    if (!out)
        return fail(FQ_ERR_NULL, "fq_plan_create_staged: out is NULL");
    *out = nullptr;
    if (!layers || !xs || !ys || !stage || !workspace)
        return fail(FQ_ERR_NULL, "fq_plan_create_staged: NULL argument");
    if (count < 1)
        return fail(FQ_ERR_SHAPE, "fq_plan_create_staged: count must be >= 1 (got %d)", count);
    if (M != 1)
        return fail(FQ_ERR_SHAPE, "fq_plan_create_staged: the stage-ordered kernel serves M = 1 (got %d)", M);
    if (stage[0] != 0)
        return fail(FQ_ERR_SHAPE, "fq_plan_create_staged: stage[0] must be 0 (got %d)", stage[0]);
    std::vector<int32_t> begin;
    begin.push_back(0);
    for (int i = 1; i < count; i++) {
        if (stage[i] != stage[i - 1] && stage[i] != stage[i - 1] + 1)
            return fail(FQ_ERR_SHAPE, "fq_plan_create_staged: stage numbers must not decrease and must rise by "
                                      "at most one (entry %d: %d after %d)", i, stage[i], stage[i - 1]);
        if (stage[i] != stage[i - 1])
            begin.push_back(i);
        if (i + 1 - begin.back() > FQ_MAX_STAGE_ENTRIES)
            return fail(FQ_ERR_SHAPE, "fq_plan_create_staged: stage %d has more than %d entries", stage[i],
                        FQ_MAX_STAGE_ENTRIES);
    }
    const int n_stages = (int)begin.size();
    begin.push_back(count);
    if (workspace_bytes < fq_plan_staged_workspace_bytes(count, n_stages))
        return fail(FQ_ERR_SHAPE, "fq_plan_create_staged: workspace too small (%zu < %zu bytes)", workspace_bytes,
                    fq_plan_staged_workspace_bytes(count, n_stages));
    if (reinterpret_cast<uintptr_t>(workspace) & 255u)
        return fail(FQ_ERR_ALIGN, "fq_plan_create_staged: workspace must be 256-byte aligned");
    std::vector<FqLinearDesc> table((size_t)count);
    FqPlanGeom geom;
    if (int rc = fq_plan_layout("fq_plan_create_staged", count, layers, xs, ys, M, table.data(), &geom))
        return rc;
    for (int a = 0; a < count; a++) // a later stage may read what an earlier one writes, never the reverse
        for (int b = 0; b < count; b++)
            if (stage[a] <= stage[b] && xs[a] == ys[b])
                return fail(FQ_ERR_SHAPE, "fq_plan_create_staged: x of entry %d (stage %d) is y of entry %d (stage %d)",
                            a, stage[a], b, stage[b]);
    const size_t lds = fq_staged_lds_bytes(n_stages, geom.max_K, STAGED_RES_CHUNKS);
    if (lds > 160 * 1024)
        return fail(FQ_ERR_SHAPE, "fq_plan_create_staged: %d stages with rows of up to %d inputs need %zu bytes of "
                                  "LDS (160 KiB at most)", n_stages, geom.max_K, lds);
    if (fq_staged_grid(lds) < 1)
        return fail(FQ_ERR_HIP, "fq_plan_create_staged: the stage-ordered kernel does not fit this device");
    fq_plan *p = new (std::nothrow) fq_plan();
    if (!p)
        return fail(FQ_ERR_HIP, "fq_plan_create_staged: out of host memory");
    char *ws = (char *)workspace;
    const size_t tb = staged_table_bytes(count), bb = staged_begin_bytes(n_stages);
    hipError_t e = hipMemcpyAsync(ws, table.data(), (size_t)count * sizeof(FqLinearDesc), hipMemcpyHostToDevice,
                                  (hipStream_t)stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(ws + tb, begin.data(), begin.size() * 4, hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e == hipSuccess) // counters and status words start at zero; every launch leaves the counters at zero
        e = hipMemsetAsync(ws + tb + bb, 0, STAGED_SYNC_BYTES, (hipStream_t)stream);
    if (e == hipSuccess)
        e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) {
        delete p;
        return hip_fail(e, "fq_plan_create_staged table copy");
    }
    p->magic = PLAN_MAGIC;
    p->geom = geom;
    p->table_dev = (const FqLinearDesc *)ws;
    p->queue_dev = nullptr;
    p->order_dev = nullptr;
    p->n_stages = n_stages;
    p->stage_begin_dev = (const int32_t *)(ws + tb);
    p->sync_dev = (int *)(ws + tb + bb);
    p->wait_limit = STAGED_WAIT_LIMIT;
    *out = p;
    return FQ_OK;
}

int fq_plan_set_wait_limit(fq_plan *plan, long long polls)
{
    if (!plan || plan->magic != PLAN_MAGIC)
        return fail(FQ_ERR_NULL, "fq_plan_set_wait_limit: plan is NULL or not valid");
    if (plan->n_stages < 1)
        return fail(FQ_ERR_SHAPE, "fq_plan_set_wait_limit: not a stage-ordered plan");
    if (polls < 0)
        return fail(FQ_ERR_SHAPE, "fq_plan_set_wait_limit: polls must be >= 0");
    plan->wait_limit = polls;
    return FQ_OK;
}

int fq_plan_status(const fq_plan *plan, int32_t *gave_up, int32_t *flags, void *stream)
{
    if (!plan || plan->magic != PLAN_MAGIC)
        return fail(FQ_ERR_NULL, "fq_plan_status: plan is NULL or not valid");
    int32_t words[2] = {0, 0}; // the sticky count of launches that gave up, then the flags
    hipError_t e = plan->n_stages < 1 // a plan of independent entries has no waits to give up
        ? hipMemcpyAsync(words + 1, plan->queue_dev + FQ_Q_FLAGS, sizeof(int32_t), hipMemcpyDeviceToHost, (hipStream_t)stream)
        : hipMemcpyAsync(words, plan->sync_dev + 1, sizeof words, hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess)
        e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_plan_status copy");
    if (gave_up)
        *gave_up = words[0];
    if (flags)
        *flags = words[1];
    return FQ_OK;
}

int fq_plan_run(const fq_plan *plan, const int32_t *bits_dev, void *stream)
{
    if (!plan || plan->magic != PLAN_MAGIC)
        return fail(FQ_ERR_NULL, "fq_plan_run: plan is NULL or not valid");
    if (!bits_dev)
        return fail(FQ_ERR_NULL, "fq_plan_run: bits_dev is NULL");
    if (reinterpret_cast<uintptr_t>(bits_dev) & 3u)
        return fail(FQ_ERR_ALIGN, "fq_plan_run: bits_dev must be 4-byte aligned");
    hipError_t e = plan->n_stages > 0
        ? fq_launch_decode_staged(plan->table_dev, bits_dev, plan->stage_begin_dev, plan->n_stages, plan->geom.max_K,
                                  STAGED_RES_CHUNKS, plan->sync_dev, plan->wait_limit, (hipStream_t)stream)
        : fq_plan_launch(plan->geom, plan->table_dev, plan->queue_dev, plan->order_dev, bits_dev,
                         (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_plan_run launch");
    return FQ_OK;
}

int fq_plan_destroy(fq_plan *plan)
{
    if (!plan || plan->magic != PLAN_MAGIC)
        return fail(FQ_ERR_NULL, "fq_plan_destroy: plan is NULL or not valid");
    plan->magic = 0;
    delete plan;
    return FQ_OK;
}

size_t fq_sched_state_bytes(int window)
{
    if (window < 1 || window > 1024)
        return 0;
    return (offsetof(FqSchedState, ring) + (size_t)window * sizeof(double) + 255) / 256 * 256;
}

int fq_sched_init(void *state, int window, double thre, int per_trigger, const int32_t *ev_entry,
                  const int32_t *ev_bits, int n_events, int32_t *bits, int entries, int32_t *ev_token, void *stream)
{
    if (!state || !bits)
        return fail(FQ_ERR_NULL, "fq_sched_init: state or bits is NULL");
    if (window < 1 || window > 1024 || per_trigger < 1 || n_events < 0 || entries < 1)
        return fail(FQ_ERR_SHAPE, "fq_sched_init: need 1 <= window <= 1024, per_trigger >= 1, "
                                  "n_events >= 0, entries >= 1 (got %d, %d, %d, %d)", window, per_trigger, n_events,
                    entries);
    if (n_events > 0 && (!ev_entry || !ev_bits))
        return fail(FQ_ERR_NULL, "fq_sched_init: ev_entry / ev_bits are NULL");
    if ((reinterpret_cast<uintptr_t>(state) & 7u) || (reinterpret_cast<uintptr_t>(bits) & 3u) ||
        (reinterpret_cast<uintptr_t>(ev_entry) & 3u) || (reinterpret_cast<uintptr_t>(ev_bits) & 3u) ||
        (reinterpret_cast<uintptr_t>(ev_token) & 3u))
        return fail(FQ_ERR_ALIGN, "fq_sched_init: state needs 8-byte, int arrays 4-byte alignment");
    hipError_t e = fq_launch_sched_init((FqSchedState *)state, window, thre, per_trigger, ev_entry,
                                        ev_bits, n_events, bits, entries, ev_token, (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_sched_init launch");
    return FQ_OK;
}

int fq_sched_threshold_from_prefill(void *state, const float *entropy, int R, int last_n, void *stream)
{
    if (!state || !entropy)
        return fail(FQ_ERR_NULL, "fq_sched_threshold_from_prefill: NULL argument");
    if (R < 1 || last_n < 1)
        return fail(FQ_ERR_SHAPE, "fq_sched_threshold_from_prefill: need R >= 1 and last_n >= 1");
    hipError_t e = fq_launch_sched_threshold((FqSchedState *)state, entropy, R, last_n, (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_sched_threshold_from_prefill launch");
    return FQ_OK;
}

int fq_sched_step(void *state, const float *entropy, void *stream)
{
    if (!state || !entropy)
        return fail(FQ_ERR_NULL, "fq_sched_step: NULL argument");
    hipError_t e = fq_launch_sched_step((FqSchedState *)state, entropy, (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_sched_step launch");
    return FQ_OK;
}

int fq_sched_peek(const void *state, int *next_event, int *tokens, double *thre, double *last_mean,
                  void *stream)
{
    if (!state)
        return fail(FQ_ERR_NULL, "fq_sched_peek: state is NULL");
    FqSchedState h;
    hipError_t e = hipMemcpyAsync(&h, state, offsetof(FqSchedState, ring), hipMemcpyDeviceToHost,
                                  (hipStream_t)stream);
    if (e == hipSuccess)
        e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_sched_peek copy");
    if (next_event)
        *next_event = h.next_event;
    if (tokens)
        *tokens = h.token;
    if (thre)
        *thre = h.thre;
    if (last_mean)
        *last_mean = h.last_mean;
    return FQ_OK;
}

int fq_entropy_kl(const float *logits_p, const float *logits_q, int R, int V, float *entropy_out,
                  float *kl_out, void *stream)
{
    if (R < 0 || V < 1)
        return fail(FQ_ERR_SHAPE, "fq_entropy_kl: need R >= 0 and V >= 1 (got R=%d V=%d)", R, V);
    if (!logits_p || !entropy_out)
        return fail(FQ_ERR_NULL, "fq_entropy_kl: logits_p or entropy_out is NULL");
    if ((logits_q == nullptr) != (kl_out == nullptr))
        return fail(FQ_ERR_NULL, "fq_entropy_kl: logits_q and kl_out must both be given or both be NULL");
    if ((reinterpret_cast<uintptr_t>(logits_p) & 3u) || (reinterpret_cast<uintptr_t>(logits_q) & 3u) ||
        (reinterpret_cast<uintptr_t>(entropy_out) & 3u) || (reinterpret_cast<uintptr_t>(kl_out) & 3u))
        return fail(FQ_ERR_ALIGN, "fq_entropy_kl: pointers must be 4-byte aligned");
    hipError_t e = fq_launch_entropy_kl(logits_p, logits_q, R, V, entropy_out, kl_out, (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_entropy_kl launch");
    return FQ_OK;
}

int fq_entropy_kl_f16(const void *logits_p, const void *logits_q, int R, int V, float *entropy_out,
                      float *kl_out, void *stream)
{
    if (R < 0 || V < 1)
        return fail(FQ_ERR_SHAPE, "fq_entropy_kl_f16: need R >= 0 and V >= 1 (got R=%d V=%d)", R, V);
    if (!logits_p || !entropy_out)
        return fail(FQ_ERR_NULL, "fq_entropy_kl_f16: logits_p or entropy_out is NULL");
    if ((logits_q == nullptr) != (kl_out == nullptr))
        return fail(FQ_ERR_NULL, "fq_entropy_kl_f16: logits_q and kl_out must both be given or both be NULL");
    if ((reinterpret_cast<uintptr_t>(logits_p) & 1u) || (reinterpret_cast<uintptr_t>(logits_q) & 1u) ||
        (reinterpret_cast<uintptr_t>(entropy_out) & 3u) || (reinterpret_cast<uintptr_t>(kl_out) & 3u))
        return fail(FQ_ERR_ALIGN, "fq_entropy_kl_f16: logits must be 2-byte and outputs 4-byte aligned");
    hipError_t e = fq_launch_entropy_kl_f16((const uint16_t *)logits_p, (const uint16_t *)logits_q, R, V,
                                            entropy_out, kl_out, (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_entropy_kl_f16 launch");
    return FQ_OK;
}

int fq_rank_ascending(const float *values, int n, int m, int32_t *order, void *stream)
{
    if (n < 0 || n > FQ_MAX_RANK_ENTRIES || m < 1 || m > FQ_MAX_RANK_ROWS)
        return fail(FQ_ERR_SHAPE, "fq_rank_ascending: need 0 <= n <= %d and 1 <= m <= %d (got n=%d m=%d)",
                    FQ_MAX_RANK_ENTRIES, FQ_MAX_RANK_ROWS, n, m);
    if (!values || !order)
        return fail(FQ_ERR_NULL, "fq_rank_ascending: values or order is NULL");
    if ((reinterpret_cast<uintptr_t>(values) & 3u) || (reinterpret_cast<uintptr_t>(order) & 3u))
        return fail(FQ_ERR_ALIGN, "fq_rank_ascending: pointers must be 4-byte aligned");
    hipError_t e = fq_launch_rank_ascending(values, n, m, order, (hipStream_t)stream);
    if (e != hipSuccess)
        return hip_fail(e, "fq_rank_ascending launch");
    return FQ_OK;
}

} // extern "C"
