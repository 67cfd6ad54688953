// Token-wise precision switching on the device, Sec. 4.4 and Alg. 1: the perplexity entropy
// PPLE = exp(entropy) of every generated token (Sec. 4.2 Eq. (5)) enters a sliding window
// (20 tokens in the paper); when the window is full and its average falls below the
// threshold, the next entries of the replacement order (ascending offline KL, Sec. 4.3) get
// their lower bit-width, and the window is emptied so that the next judgement only sees
// tokens generated at the new precision.
//
// The state, the order and the per-entry bit-width array all live in device memory and the
// step is one single-lane kernel, so a decode loop never has to bring PPLE to the host to
// decide what the next token's linears run at: the plan kernels read the same bit-width
// array.  PPLE and the average are taken in double; the average is the sum of the window's
// slots in slot order divided by the window length.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "fq_internal.h"

__global__ void sched_init_kernel(FqSchedState *s, int window, double thre, int per_trigger,
                                  const int32_t *ev_entry, const int32_t *ev_bits, int n_events,
                                  int32_t *bits, int entries, int32_t *ev_token)
{
    if (threadIdx.x != 0 || blockIdx.x != 0)
        return;
    s->thre = thre;
    s->last_mean = 0.0;
    s->window = window;
    s->per_trigger = per_trigger;
    s->n_events = n_events;
    s->next_event = 0;
    s->pos = 0;
    s->count = 0;
    s->token = 0;
    s->entries = entries;
    s->ev_entry = ev_entry;
    s->ev_bits = ev_bits;
    s->bits = bits;
    s->ev_token = ev_token;
    for (int i = 0; i < window; i++)
        s->ring[i] = 0.0;
}

// thre <- mean PPLE of the last `last_n` of R prefill positions (Alg. 1)
__global__ void sched_threshold_kernel(FqSchedState *s, const float *entropy, int R, int last_n)
{
    if (threadIdx.x != 0 || blockIdx.x != 0)
        return;
    if (last_n > R)
        last_n = R;
    double sum = 0.0;
    for (int r = R - last_n; r < R; r++)
        sum += exp((double)entropy[r]);
    s->thre = sum / (double)last_n;
}

__global__ void sched_step_kernel(FqSchedState *s, const float *entropy)
{
    if (threadIdx.x != 0 || blockIdx.x != 0)
        return;
    const double pple = exp((double)entropy[0]);
    const int window = s->window;
    int pos = s->pos, count = s->count;
    s->ring[pos] = pple;
    pos = pos + 1 == window ? 0 : pos + 1;
    if (count < window)
        count++;
    if (count == window) {
        double sum = 0.0;
        for (int i = 0; i < window; i++)
            sum += s->ring[i];
        const double mean = sum / (double)window;
        s->last_mean = mean;
        int next = s->next_event;
        if (mean < s->thre && next < s->n_events) {
            for (int j = 0; j < s->per_trigger && next < s->n_events; j++) {
                // an event that names no entry of the array, or no bit-width, is passed over (a
                // replacement order ranked over another number of linears must not write beside
                // the array the plan reads)
                const int e = s->ev_entry[next], b = s->ev_bits[next];
                const bool ok = e >= 0 && e < s->entries && (b == 2 || b == 3 || b == 4 || b == 8 || b == 16);
                if (ok)
                    s->bits[e] = b;
                if (s->ev_token)
                    s->ev_token[next] = ok ? s->token : -2;
                next++;
            }
            s->next_event = next;
            count = 0; // judge again only after a full window at the new precision
        }
    }
    s->pos = pos;
    s->count = count;
    s->token = s->token + 1;
}

hipError_t fq_launch_sched_init(FqSchedState *s, int window, double thre, int per_trigger,
                                const int32_t *ev_entry, const int32_t *ev_bits, int n_events,
                                int32_t *bits, int entries, int32_t *ev_token, hipStream_t stream)
{
    sched_init_kernel<<<1, 64, 0, stream>>>(s, window, thre, per_trigger, ev_entry, ev_bits, n_events,
                                           bits, entries, ev_token);
    return hipGetLastError();
}

hipError_t fq_launch_sched_threshold(FqSchedState *s, const float *entropy, int R, int last_n,
                                     hipStream_t stream)
{
    sched_threshold_kernel<<<1, 64, 0, stream>>>(s, entropy, R, last_n);
    return hipGetLastError();
}

hipError_t fq_launch_sched_step(FqSchedState *s, const float *entropy, hipStream_t stream)
{
    sched_step_kernel<<<1, 64, 0, stream>>>(s, entropy);
    return hipGetLastError();
}

// Replacement order of Sec. 4.3: entries sorted by ascending KL divergence.  The key of entry
// e is the sum of its m values (KL on m calibration rows) in double, in index order.
// Rank by counting: the place of an entry is the number of entries that come before it
// (smaller key; equal keys in index order; NaN keys after every number), so every place is
// written exactly once without any exchange between workgroups.  Keys are recomputed tile by
// tile into LDS: n is the number of linears of a model, a few hundred.
constexpr int RANK_THREADS = 256;

__global__ __launch_bounds__(RANK_THREADS) void rank_ascending_kernel(const float *__restrict__ values,
                                                                      int n, int m,
                                                                      int32_t *__restrict__ order)
{
    __shared__ double s_key[RANK_THREADS];
    const int e = blockIdx.x * RANK_THREADS + threadIdx.x;
    auto key_of = [&](int i) {
        double k = 0.0;
        for (int j = 0; j < m; j++)
            k += (double)values[(size_t)i * m + j];
        return k;
    };
    const double mine = e < n ? key_of(e) : 0.0;
    const bool mine_nan = mine != mine;
    int before = 0;
    for (int base = 0; base < n; base += RANK_THREADS) {
        const int other = base + threadIdx.x;
        __syncthreads(); // the previous tile has been read by everyone
        s_key[threadIdx.x] = other < n ? key_of(other) : 0.0;
        __syncthreads();
        const int cnt = min(RANK_THREADS, n - base);
        for (int t = 0; t < cnt; t++) {
            const double k = s_key[t];
            const int idx = base + t;
            const bool k_nan = k != k;
            bool first; // does entry idx come before entry e?
            if (k_nan != mine_nan)
                first = mine_nan;
            else if (k_nan || k == mine)
                first = idx < e;
            else
                first = k < mine;
            before += first ? 1 : 0;
        }
    }
    if (e < n)
        order[before] = e;
}

hipError_t fq_launch_rank_ascending(const float *values, int n, int m, int32_t *order,
                                    hipStream_t stream)
{
    if (n == 0)
        return hipSuccess;
    rank_ascending_kernel<<<(n + RANK_THREADS - 1) / RANK_THREADS, RANK_THREADS, 0, stream>>>(values, n, m,
                                                                                               order);
    return hipGetLastError();
}
