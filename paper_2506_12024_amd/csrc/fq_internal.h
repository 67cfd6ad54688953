// Internal declarations shared by the host API and the kernel files.
#ifndef FQ_INTERNAL_H
#define FQ_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

// One linear of a launch: which resident copies exist and where x and y live.
// Plain data, passed by value in the kernel arguments (single call) or read
// from a device table (plan).
struct FqLinearDesc {
    const uint8_t *codes4;  // [N][K/2] or null
    const float *scales4;   // [N][K/128]
    const uint8_t *zeros4;  // [N][K/128]
    const uint8_t *codes8;  // [N][K] or null
    const float *scales8;
    const uint8_t *zeros8;
    const uint16_t *w16;    // fp16 [N][K] or null
    const uint8_t *codes2;  // [N][K/4] or null (not served by the streaming batch kernel and the GEMM)
    const float *scales2;
    const uint8_t *zeros2;
    const uint8_t *codes3;  // [N][K/32] blocks of 12 bytes, or null (not served by the streaming batch kernel and the GEMM)
    const float *scales3;
    const uint8_t *zeros3;
    const uint16_t *x;      // fp16 [M][K]
    uint16_t *y;            // fp16 [M][N]
    int N;
    int K;
    int tile_begin;         // first row tile of this entry in the plan's global tile numbering
    int pad;
};

// Geometry of a plan: how its entries are cut into row tiles for the kernel that serves its M.
struct FqPlanGeom {
    int count, M, total_tiles, tile_rows, max_K;
    int has3; // some layer of the plan holds a 3-bit copy
};
struct fq_layer;
// Records a message for fq_last_error() on the calling thread and returns `code`.
int fq_fail(int code, const char *fmt, ...);
// Argument checks and layout shared by the entry points that run a list of linears with one launch:
// fills table[count] and *geom, or returns a negative fq_status with the message recorded.
int fq_plan_layout(const char *who, int count, const fq_layer *const *layers, const void *const *xs,
                   void *const *ys, int M, FqLinearDesc *table, FqPlanGeom *geom);
// The launch of a laid-out plan whose table, queue words and entry list are in device memory.
hipError_t fq_plan_launch(const FqPlanGeom &g, const FqLinearDesc *table_dev, int *queue_dev, void *order_dev,
                          const int32_t *bits_dev, hipStream_t stream);

// Facts about the current device, asked of the runtime once per device and cached (thread-safe):
// its compute units; the workgroups of `func` (launched with `threads` threads and `lds` bytes of
// dynamic LDS) that fit on one of them, `fallback` if the runtime cannot say; and a kernel's
// dynamic LDS limit raised to at least `bytes` (a no-op once done).
int fq_device_cus();
int fq_workgroups_per_cu(const void *func, int threads, size_t lds, int fallback);
hipError_t fq_raise_dynamic_lds(const void *func, size_t bytes);
// The kernels that combine the partial results of their workgroups through a static device array
// (entropy / KL over a few long rows, the fused output layer) keep FQ_BANKS copies of it,
// one per stream: calls on different streams then never share one.  The bank of `stream` on the
// current device (the first FQ_BANKS distinct streams get one each), or -1 if none is left.
constexpr int FQ_BANKS = 16; // FQ_SCRATCH_BANKS of the public header
int fq_stream_bank(hipStream_t stream);

hipError_t fq_launch_quantize(const void *w, long long n_groups, int bits, bool symmetric, void *codes,
                              void *scales, void *zeros, hipStream_t stream);
// 8 bits, one group per row (group = K)
hipError_t fq_launch_quantize_row8(const void *w, int N, int K, bool symmetric, void *codes, void *scales, void *zeros,
                                   hipStream_t stream);
hipError_t fq_launch_fake_quantize(const void *w, long long n_groups, int bits, bool symmetric, void *w_hat,
                                   hipStream_t stream);

hipError_t fq_launch_entropy_kl(const float *a, const float *b, int R, int V, float *H, float *KL,
                                hipStream_t stream);

hipError_t fq_launch_entropy_kl_f16(const uint16_t *a, const uint16_t *b, int R, int V, float *H,
                                    float *KL, hipStream_t stream);

// Skinny (decode) linears.  `descs` is a device table of `count` entries when
// `single` is null, else the one entry is passed by value and bits_host applies.
// `flags` (plans; may be null): a device word that gets bit 0 set when an entry could not be served.
hipError_t fq_launch_decode(const FqLinearDesc *single, int bits_host,
                            const FqLinearDesc *descs_dev, const int32_t *bits_dev, int count,
                            int total_tiles, int tile_rows, int max_K, int M, int *flags, hipStream_t stream);
// Rows per tile (multiple of 16) for a launch that covers `total_rows` output rows.
int fq_decode_tile_rows(long long total_rows, int max_K, int M);

// Stage-ordered plan at M = 1 in one persistent launch: entries [stage_begin[s], stage_begin[s + 1])
// form stage s; `sync_dev` holds the barrier's counters and status words (zero before the first
// launch).  fq_staged_lds_bytes: dynamic LDS the kernel needs; fq_staged_grid: workgroups it is
// launched with (0 = does not fit the current device).
size_t fq_staged_lds_bytes(int n_stages, int max_K, int res_chunks);
int fq_staged_grid(size_t lds_bytes);
// Bytes of a stage-ordered plan's sync words: status words, then the arrival counters of the barrier.
constexpr size_t FQ_STAGED_SYNC_BYTES = 32768;
hipError_t fq_launch_decode_staged(const FqLinearDesc *table_dev, const int32_t *bits_dev,
                                   const int32_t *stage_begin_dev, int n_stages, int max_K, int res_chunks,
                                   int *sync_dev, long long wait_limit, hipStream_t stream);

// Same contract for 2 <= M <= 32 (MFMA skinny kernel); tile rows are 16 (K split), 64, 128 or 256.
// with3: the launch may meet a 3-bit entry (the instance with the 3-bit path, which costs registers)
hipError_t fq_launch_skinny(const FqLinearDesc *single, int bits_host,
                            const FqLinearDesc *descs_dev, const int32_t *bits_dev, int count,
                            int total_tiles, int tile_rows, int M, bool with3, int *queue, void *order,
                            hipStream_t stream);
int fq_skinny_tile_rows(long long total_rows, int M);
// Streaming variant for plan launches with 2 <= M <= 32 and tiles of 256 rows (fq_launch_skinny
// hands those to it).
hipError_t fq_launch_skinny_stream(const FqLinearDesc *descs_dev, const int32_t *bits_dev, int count,
                                   int total_tiles, int M, int cus, int *queue, void *order, hipStream_t stream);
// The plan's queue words (ints): a tile cursor per XCD, the count of workgroups that have finished,
// then what plan_order_kernel leaves for the launch that follows it: tiles and entries of the
// streaming kernel's list.
constexpr int FQ_Q_DONE = 8, FQ_Q_TILES = 9, FQ_Q_ENTRIES = 10;
// ... and, apart from those, a sticky word of flags that fq_plan_status reports: bit 0 = an entry's
// bit-width was not one the plan serves, or had no copy attached, in some run (its y was left untouched)
constexpr int FQ_Q_FLAGS = 16;

// Device-resident state of the precision scheduler (ring of PPLE values follows the header).
struct FqSchedState {
    double thre;
    double last_mean;
    int window, per_trigger, n_events, next_event, pos, count, token, entries;
    const int32_t *ev_entry;
    const int32_t *ev_bits;
    int32_t *bits;
    int32_t *ev_token;
    double ring[1]; // `window` slots
};
hipError_t fq_launch_sched_init(FqSchedState *s, int window, double thre, int per_trigger,
                                const int32_t *ev_entry, const int32_t *ev_bits, int n_events,
                                int32_t *bits, int entries, int32_t *ev_token, hipStream_t stream);
hipError_t fq_launch_sched_threshold(FqSchedState *s, const float *entropy, int R, int last_n,
                                     hipStream_t stream);
hipError_t fq_launch_sched_step(FqSchedState *s, const float *entropy, hipStream_t stream);

hipError_t fq_launch_rank_ascending(const float *values, int n, int m, int32_t *order,
                                    hipStream_t stream);

// Prefill-shaped dequant-GEMM on MFMA.
hipError_t fq_launch_prefill(const FqLinearDesc &d, int bits, int M, hipStream_t stream);


// W8A8 prefill: per-token symmetric 8-bit activation quantization (also writes the per-group
// code sums, [K/128][M]) and the int8 MFMA GEMM against the resident 8-bit copy.
hipError_t fq_launch_quantize_act(const void *x, int M, int K, void *xq, float *sx, int32_t *xsum,
                                  hipStream_t stream);
// per_row: the 8-bit copy has one scale and zero point per weight row (group = K) instead of per 128 inputs
hipError_t fq_launch_w8a8(const FqLinearDesc &d, const void *xq, const float *sx, const int32_t *xsum,
                          int M, bool per_row, hipStream_t stream);

// Output layer (fp16 weight [V][K], 1 <= M <= 4 rows of x) fused with entropy and argmax of its logits.
hipError_t fq_launch_lm_head_entropy(const void *x, const void *w, int M, int V, int K, float *logits, float *H,
                                     int32_t *argmax, hipStream_t stream);

#endif
