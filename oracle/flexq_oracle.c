/*
 * CPU oracle for the FlexQuant decode hot path.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product library includes, links or calls this file; it
 * exists so that the GPU kernels can be checked against a plain, slow,
 * obviously correct statement of what the paper defines.
 *
 * Written from the paper's definitions, one routine per definition:
 *   orc_quantize     asymmetric uniform quantization, Sec. 2.2 Eq. (2), applied
 *                    per (output row, group of `group` consecutive inputs)
 *   orc_dequant      Sec. 2.2 Eq. (3)
 *   orc_linear       the weight-only quantized linear layer of the decode
 *                    phase (Sec. 4.1, 4.3): y = x . dequant(W)^T
 *   orc_entropy_kl   softmax of Sec. 2.3, the entropy inside the perplexity
 *                    entropy of Sec. 4.2 Eq. (5), and the KL divergence of
 *                    Sec. 3.1 between two next-token distributions
 *   orc_sched_*      token-wise precision switching, Sec. 4.4 and Alg. 1
 *   orc_rank_ascending   the replacement order of Sec. 4.3 (ascending KL)
 *   orc_quantize_act, orc_linear_w8a8   the W8A8 prefill of Sec. 4.1 / 4.3 / 4.5
 *
 * Readings taken where the paper is silent (kept in step with the design
 * notes of this repository):
 *   - statistics Xmin/Xmax are per (row, group); the range is widened to
 *     contain 0 so that the zero point fits the code range;
 *   - the bracket of Eq. (2) is round-half-to-even; s, z and the codes are
 *     computed in binary32 with one rounding per operation (no fused
 *     multiply-add, true division);
 *   - Eq. (2)'s X/s + z is added first and rounded second, then clamped to
 *     [0, 2^n - 1]; an all-zero group gets s = 1, z = 0;
 *   - packing: 8-bit codes one per byte; 4-bit codes two per byte, even
 *     input index in the low nibble;
 *   - the sum of Eq. (5) runs over the vocabulary, natural logarithm,
 *     0 log 0 = 0; KL(p || q) takes p from the first logits vector.
 *
 * Everything that accumulates does so in double.  No blocking, no fusion.
 * Build: gcc -O2 -ffp-contract=off (and -fopenmp: rows of orc_linear and of
 * orc_entropy_kl may run on several threads; each output is still computed by
 * one thread in index order).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- binary16 <-> binary32/64, written out (no compiler half type) ---- */

static float half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    int e = (h >> 10) & 0x1F;
    uint32_t m = h & 0x3FFu;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m | 0x400u), e - 25);
    float f = (float)v; /* exact: every half is a float */
    if (sign)
        f = -f;
    return f;
}

/* double -> nearest binary16 (ties to even), by explicit search of the two
 * neighbouring halves; overflow beyond the rounding boundary gives infinity. */
static uint16_t double_to_half(double d)
{
    uint16_t sign = 0;
    if (isnan(d))
        return 0x7E00u;
    if (d < 0 || (d == 0 && signbit(d))) {
        sign = 0x8000u;
        d = -d;
    }
    if (d >= 65520.0)
        return (uint16_t)(sign | 0x7C00u);
    /* largest half <= d by bisection over the ordered bit patterns 0..0x7BFF */
    uint16_t lo = 0, hi = 0x7BFF;
    while (lo < hi) {
        uint16_t mid = (uint16_t)((lo + hi + 1) >> 1);
        if ((double)half_to_float(mid) <= d)
            lo = mid;
        else
            hi = (uint16_t)(mid - 1);
    }
    double below = (double)half_to_float(lo);
    double above = (lo == 0x7BFF) ? 65536.0 : (double)half_to_float((uint16_t)(lo + 1));
    double dl = d - below, du = above - d; /* both exact in double */
    uint16_t r;
    if (dl < du)
        r = lo;
    else if (dl > du)
        r = (uint16_t)(lo + 1);
    else
        r = (lo & 1u) ? (uint16_t)(lo + 1) : lo;
    return (uint16_t)(sign | r);
}

float orc_half_to_float(uint16_t h) { return half_to_float(h); }
uint16_t orc_double_to_half(double d) { return double_to_half(d); }

/* ---- Eq. (2): quantize one matrix, group-wise along the input dimension ---- */

/* Packed codes: 8 bits one per byte; 4 bits two per byte, the even k in the low nibble; 2 bits
 * four per byte, k % 4 = 0 in bits 0..1 up to k % 4 = 3 in bits 6..7.  Rows follow each other.
 * 3 bits (the paper names no format for its 3-bit models; this is the repository's): a row is
 * K / 32 blocks of 12 bytes, block b holding k = 32 b .. 32 b + 31, read as three little-endian
 * 32-bit words.  Word j holds codes 10 j .. 10 j + 9 whole: code 10 j + 5 h + p (h = 0, 1;
 * p = 0 .. 4) in bits 16 h + 3 p .. 16 h + 3 p + 2.  That leaves bit 15 and bit 31 of every word:
 * bit 15 of word t is bit t of code 30, bit 31 of word t is bit t of code 31. */
static int bit_place3(int i, int t) /* where bit t of code i of a block sits among the block's 96 bits */
{
    if (i < 30)
        return 32 * (i / 10) + 16 * ((i % 10) / 5) + 3 * (i % 5) + t;
    return 32 * t + 15 + 16 * (i - 30);
}

static int code_of(const uint8_t *codes, int bits, long long row_elems, long long n, long long k)
{
    if (bits == 3) {
        const uint8_t *blk = codes + n * (row_elems * 3 / 8) + (k / 32) * 12;
        int q = 0;
        for (int t = 0; t < 3; t++) {
            const int place = bit_place3((int)(k % 32), t);
            q |= ((blk[place / 8] >> (place % 8)) & 1) << t;
        }
        return q;
    }
    if (bits == 8)
        return codes[n * row_elems + k];
    if (bits == 2)
        return (codes[(n * row_elems + k) / 4] >> (2 * (k & 3))) & 3;
    uint8_t byte = codes[(n * row_elems + k) / 2];
    return (k & 1) ? (byte >> 4) : (byte & 0xF);
}

static void put_code(uint8_t *codes, int bits, long long row_elems, long long n, long long k, unsigned q)
{
    if (bits == 3) {
        uint8_t *blk = codes + n * (row_elems * 3 / 8) + (k / 32) * 12;
        for (int t = 0; t < 3; t++) {
            const int place = bit_place3((int)(k % 32), t);
            blk[place / 8] |= (uint8_t)(((q >> t) & 1u) << (place % 8));
        }
        return;
    }
    if (bits == 8)
        codes[n * row_elems + k] = (uint8_t)q;
    else if (bits == 2)
        codes[(n * row_elems + k) / 4] |= (uint8_t)(q << (2 * (k & 3)));
    else
        codes[(n * row_elems + k) / 2] |= (uint8_t)(q << ((k & 1) ? 4 : 0));
}

/*
 * w: [N][K] binary16 bit patterns.  codes: N*K*bits/8 bytes.  scales: [N][K/group]
 * float.  zeros: [N][K/group] bytes.  Returns 0, or -1 on a bad argument
 * (bits not 2, 3, 4 or 8, K not a multiple of group, an odd group, at 2 bits a group that is not a
 * multiple of 4, at 3 bits one that is not a multiple of 32) or a non-finite weight.
 */
int orc_quantize(const uint16_t *w, int N, int K, int bits, int group,
                 uint8_t *codes, float *scales, uint8_t *zeros)
{
    if ((bits != 2 && bits != 3 && bits != 4 && bits != 8) || group <= 0 || (group & 1) || (bits == 2 && (group & 3)) ||
        (bits == 3 && (group & 31)) || K % group != 0)
        return -1;
    const int G = K / group;
    const float qmax = (float)((1 << bits) - 1);
    int bad = 0;
    if (bits != 8)
        memset(codes, 0, (size_t)N * K * bits / 8);
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (long long n = 0; n < N; n++) {
        for (int g = 0; g < G; g++) {
            const uint16_t *wg = w + n * K + (long long)g * group;
            float lo = 0.0f, hi = 0.0f; /* range always contains 0 */
            for (int i = 0; i < group; i++) {
                float v = half_to_float(wg[i]);
                if (!isfinite(v))
                    bad |= 1;
                if (v < lo) lo = v;
                if (v > hi) hi = v;
            }
            float s, zf;
            if (hi == lo) { /* all-zero group */
                s = 1.0f;
                zf = 0.0f;
            } else {
                volatile float range = hi - lo;       /* one rounding each; the   */
                volatile float sv = range / qmax;     /* volatiles forbid folding */
                s = sv;
                volatile float neg = -lo;
                volatile float zq = neg / s;
                zf = rintf(zq);                        /* q_min = 0 */
                if (zf < 0.0f) zf = 0.0f;
                if (zf > qmax) zf = qmax;
            }
            scales[n * G + g] = s;
            zeros[n * G + g] = (uint8_t)zf;
            for (int i = 0; i < group; i++) {
                float v = half_to_float(wg[i]);
                volatile float t = v / s;
                volatile float u = t + zf;
                float q = rintf(u);
                if (q < 0.0f) q = 0.0f;
                if (q > qmax) q = qmax;
                put_code(codes, bits, K, n, (long long)g * group + i, (unsigned)q);
            }
        }
    }
    return bad ? -1 : 0;
}

/*
 * Symmetric variant, stated after Sec. 2.2 Eq. (3): z = 0, Xmax = -Xmin = max |X|, and the range
 * Qmax - Qmin = 2^n - 2, i.e. integers -(2^(n-1) - 1) .. 2^(n-1) - 1.  Per group:
 * s = (2 max|w|) / (2^n - 2), q = clamp(rint(w / s)).  The result is written in the layout of
 * orc_quantize -- stored code = q + 2^(n-1), stored zero point = 2^(n-1) for every group -- so that
 * Eq. (3), s * (code - zero), gives s * q and orc_dequant / orc_linear apply unchanged.
 * An all-zero group takes s = 1.  Binary32, one rounding per operation.
 */
static float sym_scale(const uint16_t *wg, int group, int bits, int *bad)
{
    float amax = 0.0f;
    for (int i = 0; i < group; i++) {
        float v = half_to_float(wg[i]);
        if (!isfinite(v))
            *bad |= 1;
        float a = fabsf(v);
        if (a > amax) amax = a;
    }
    if (amax == 0.0f)
        return 1.0f;
    const float levels = (float)((1 << bits) - 2);
    volatile float range = amax + amax;
    volatile float sv = range / levels;
    return sv;
}

static float sym_code(float v, float s, int bits)
{
    const float lim = (float)((1 << (bits - 1)) - 1);
    volatile float t = v / s;
    float q = rintf(t);
    if (q < -lim) q = -lim;
    if (q > lim) q = lim;
    return q;
}

int orc_quantize_sym(const uint16_t *w, int N, int K, int bits, int group,
                     uint8_t *codes, float *scales, uint8_t *zeros)
{
    if ((bits != 2 && bits != 3 && bits != 4 && bits != 8) || group <= 0 || (group & 1) || (bits == 2 && (group & 3)) ||
        (bits == 3 && (group & 31)) || K % group != 0)
        return -1;
    const int G = K / group;
    const int offset = 1 << (bits - 1);
    int bad = 0;
    if (bits != 8)
        memset(codes, 0, (size_t)N * K * bits / 8);
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (long long n = 0; n < N; n++) {
        for (int g = 0; g < G; g++) {
            const uint16_t *wg = w + n * K + (long long)g * group;
            int b = 0;
            const float s = sym_scale(wg, group, bits, &b);
            bad |= b;
            scales[n * G + g] = s;
            zeros[n * G + g] = (uint8_t)offset;
            for (int i = 0; i < group; i++) {
                int q = (int)sym_code(half_to_float(wg[i]), s, bits) + offset;
                put_code(codes, bits, K, n, (long long)g * group + i, (unsigned)q);
            }
        }
    }
    return bad ? -1 : 0;
}

/*
 * Quantize and dequantize in one go, the way the paper obtained its 2-, 3- and 4-bit results
 * (Sec. 5.1: those widths were simulated, Table 1): w_hat = half(s * (q - z)) per Eq. (2) and
 * Eq. (3), bits = 2 .. 8, asymmetric (sym = 0: s, z and q exactly as in orc_quantize) or the
 * symmetric variant (sym = 1: as in orc_quantize_sym).  w_hat: [N][K] binary16 bit patterns.
 */
int orc_fake_quantize(const uint16_t *w, int N, int K, int bits, int group, int sym, uint16_t *w_hat)
{
    if (bits < 2 || bits > 8 || group <= 0 || K % group != 0)
        return -1;
    const int G = K / group;
    const float qmax = (float)((1 << bits) - 1);
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (long long n = 0; n < N; n++) {
        for (int g = 0; g < G; g++) {
            const uint16_t *wg = w + n * K + (long long)g * group;
            uint16_t *og = w_hat + n * K + (long long)g * group;
            if (sym) {
                int b = 0;
                const float s = sym_scale(wg, group, bits, &b);
                bad |= b;
                for (int i = 0; i < group; i++) {
                    const int q = (int)sym_code(half_to_float(wg[i]), s, bits); /* an integer code: no -0 */
                    volatile float d = (float)q * s;
                    og[i] = double_to_half((double)d);
                }
                continue;
            }
            float lo = 0.0f, hi = 0.0f; /* range always contains 0 */
            for (int i = 0; i < group; i++) {
                float v = half_to_float(wg[i]);
                if (!isfinite(v))
                    bad |= 1;
                if (v < lo) lo = v;
                if (v > hi) hi = v;
            }
            float s, zf;
            if (hi == lo) {
                s = 1.0f;
                zf = 0.0f;
            } else {
                volatile float range = hi - lo;
                volatile float sv = range / qmax;
                s = sv;
                volatile float neg = -lo;
                volatile float zq = neg / s;
                zf = rintf(zq);
                if (zf < 0.0f) zf = 0.0f;
                if (zf > qmax) zf = qmax;
            }
            for (int i = 0; i < group; i++) {
                float v = half_to_float(wg[i]);
                volatile float t = v / s;
                volatile float u = t + zf;
                float q = rintf(u);
                if (q < 0.0f) q = 0.0f;
                if (q > qmax) q = qmax;
                const int code = (int)q; /* what orc_quantize stores: an integer, no -0 */
                volatile float dq = (float)code - zf;
                volatile float d = dq * s;
                og[i] = double_to_half((double)d);
            }
        }
    }
    return bad ? -1 : 0;
}

/* ---- Eq. (3): dequantize to float, [N][K] ---- */

void orc_dequant(const uint8_t *codes, const float *scales, const uint8_t *zeros,
                 int N, int K, int bits, int group, float *w_hat)
{
    const int G = K / group;
    for (long long n = 0; n < N; n++)
        for (long long k = 0; k < K; k++) {
            int g = (int)(k / group);
            float q = (float)code_of(codes, bits, K, n, k);
            float z = (float)zeros[n * G + g];
            volatile float d = q - z;
            w_hat[n * K + k] = d * scales[n * G + g];
        }
}

/*
 * Weight-only quantized linear.  x: [M][K] half bits.  bits 2/4/8: codes, scales,
 * zeros as written by orc_quantize; bits 16: `codes` holds [N][K] half weights,
 * scales/zeros unused.  Rows row0 .. row0+rows-1 of the output are computed
 * (rows = N, row0 = 0 for all); y: [M][rows] half bits, y[m][n-row0].
 * Each output: sum over k in index order of (double)x * (double)w_hat, with
 * w_hat the binary32 value of Eq. (3); rounded once to binary16.
 */
int orc_linear(const uint16_t *x, int M, const uint8_t *codes, const float *scales,
               const uint8_t *zeros, int N, int K, int bits, int group,
               int row0, int rows, uint16_t *y)
{
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8 && bits != 16)
        return -1;
    if (bits != 16 && (group <= 0 || K % group != 0))
        return -1;
    if (row0 < 0 || rows < 0 || row0 + rows > N)
        return -1;
    const int G = (bits == 16) ? 0 : K / group;
#pragma omp parallel for schedule(static)
    for (long long r = 0; r < rows; r++) {
        long long n = row0 + r;
        for (int m = 0; m < M; m++) {
            double acc = 0.0;
            for (long long k = 0; k < K; k++) {
                float wv;
                if (bits == 16) {
                    wv = half_to_float(((const uint16_t *)codes)[n * K + k]);
                } else {
                    int g = (int)(k / group);
                    float q = (float)code_of(codes, bits, K, n, k);
                    float z = (float)zeros[n * G + g];
                    volatile float d = q - z;
                    volatile float p = d * scales[n * G + g];
                    wv = p;
                }
                acc += (double)half_to_float(x[(long long)m * K + k]) * (double)wv;
            }
            y[(long long)m * rows + r] = double_to_half(acc);
        }
    }
    return 0;
}

/*
 * Entropy of softmax(a) and KL(softmax(a) || softmax(b)) per row, in nats.
 * a, b: [R][V] float (b may be NULL: only the entropy is written).
 * Two passes per row, in double: m = max a; S = sum exp(a - m);
 * LSE = m + ln S; p_i = exp(a_i - m) / S; H = - sum p_i ln p_i with
 * ln p_i = a_i - LSE; KL = sum p_i (ln p_i - ln q_i).  Terms with p_i = 0 add 0.
 */
int orc_entropy_kl(const float *a, const float *b, int R, int V, double *H, double *KL)
{
    if (R < 0 || V < 1)
        return -1;
#pragma omp parallel for schedule(static)
    for (long long r = 0; r < R; r++) {
        const float *ar = a + r * V;
        const float *br = b ? b + r * V : 0;
        double ma = -INFINITY, mb = -INFINITY;
        for (int i = 0; i < V; i++) {
            if ((double)ar[i] > ma) ma = ar[i];
            if (br && (double)br[i] > mb) mb = br[i];
        }
        double Sa = 0.0, Sb = 0.0;
        for (int i = 0; i < V; i++) {
            Sa += exp((double)ar[i] - ma);
            if (br) Sb += exp((double)br[i] - mb);
        }
        double lse_a = ma + log(Sa), lse_b = br ? mb + log(Sb) : 0.0;
        double h = 0.0, kl = 0.0;
        for (int i = 0; i < V; i++) {
            double p = exp((double)ar[i] - ma) / Sa;
            if (p == 0.0)
                continue;
            double lnp = (double)ar[i] - lse_a;
            h -= p * lnp;
            if (br)
                kl += p * (lnp - ((double)br[i] - lse_b));
        }
        H[r] = h;
        if (br && KL)
            KL[r] = kl;
    }
    return 0;
}

/* ---- Token-wise precision switching, Sec. 4.4 and Alg. 1 ---------------------------
 *
 * The steps of Alg. 1's decode loop that FlexQuant adds, in the paper's order:
 *   PPLE <- exp(entropy(logits))                              (Sec. 4.2 Eq. (5))
 *   push PPLE into a sliding window of `window` generated tokens (20 in the paper)
 *   if the window is full and its average is below `thre`:
 *       replace the weights of the next layers in the offline (KL-sorted) order by
 *       their lower bit-width                                  (Sec. 4.3)
 *       and wait until a full window of tokens has been generated at the new
 *       precision before judging again                         (Sec. 4.5, last paragraph)
 *
 * Readings: the replacement order is an explicit list of events (entry, new bit-width)
 * -- ascending KL for INT8 -> INT4, or a longer ladder FP16 -> INT8 -> INT4 --, a
 * trigger applies the next `per_trigger` events, "wait for enough tokens" means the
 * window is emptied at a switch.  PPLE and the average are taken in double; the average
 * is the sum of the window's slots in slot order divided by `window`.
 */
typedef struct orc_sched {
    double thre;
    double last_mean;
    int window, per_trigger, n_events, next_event, pos, count, token;
    const int32_t *ev_entry;
    const int32_t *ev_bits;
    int32_t *bits;     /* per-entry bit-widths, updated in place */
    int32_t *ev_token; /* out: token index at which each event fired (may be NULL) */
    double ring[1024];
} orc_sched;

int orc_sched_size(void) { return (int)sizeof(orc_sched); }

int orc_sched_init(orc_sched *s, int window, double thre, int per_trigger, const int32_t *ev_entry,
                   const int32_t *ev_bits, int n_events, int32_t *bits, int32_t *ev_token)
{
    if (window < 1 || window > 1024 || per_trigger < 1 || n_events < 0)
        return -1;
    memset(s, 0, sizeof *s);
    s->thre = thre;
    s->window = window;
    s->per_trigger = per_trigger;
    s->n_events = n_events;
    s->ev_entry = ev_entry;
    s->ev_bits = ev_bits;
    s->bits = bits;
    s->ev_token = ev_token;
    return 0;
}

/* thre <- average PPLE of the last `last_n` of R prefill positions (Alg. 1, line "thre <-") */
void orc_sched_threshold_from_prefill(orc_sched *s, const float *entropy, int R, int last_n)
{
    if (last_n > R)
        last_n = R;
    double sum = 0.0;
    for (int r = R - last_n; r < R; r++)
        sum += exp((double)entropy[r]);
    s->thre = sum / (double)last_n;
}

/* One generated token whose next-token entropy is `entropy` (nats).  Returns the number of
 * events applied (0 if no switch happened). */
int orc_sched_step(orc_sched *s, float entropy)
{
    const double pple = exp((double)entropy);
    s->ring[s->pos] = pple;
    s->pos = (s->pos + 1) % s->window;
    if (s->count < s->window)
        s->count++;
    int applied = 0;
    if (s->count == s->window) {
        double sum = 0.0;
        for (int i = 0; i < s->window; i++)
            sum += s->ring[i];
        s->last_mean = sum / (double)s->window;
        if (s->last_mean < s->thre && s->next_event < s->n_events) {
            for (int j = 0; j < s->per_trigger && s->next_event < s->n_events; j++) {
                s->bits[s->ev_entry[s->next_event]] = s->ev_bits[s->next_event];
                if (s->ev_token)
                    s->ev_token[s->next_event] = s->token;
                s->next_event++;
                applied++;
            }
            s->count = 0; /* judge again only after a full window at the new precision */
        }
    }
    s->token++;
    return applied;
}

double orc_sched_thre(const orc_sched *s) { return s->thre; }
double orc_sched_last_mean(const orc_sched *s) { return s->last_mean; }
int orc_sched_next_event(const orc_sched *s) { return s->next_event; }

/*
 * The output layer followed by what Alg. 1 takes from its logits in every decode step: the
 * next token (argmax) and the entropy behind PPLE (Sec. 4.2 Eq. 5; softmax as in Sec. 2.3).
 * x: [M][K] half bits; w: [V][K] half bits (the fp16 output-layer weight).
 * logits[m][v] = sum_k x[m][k] * w[v][k] in double (optional output, may be NULL),
 * H[m] = -sum_v p ln p with p = softmax(logits[m]), argmax[m] = the smallest v that attains the
 * maximum logit.
 */
int orc_lm_head_entropy(const uint16_t *x, const uint16_t *w, int M, int V, int K, double *logits,
                        double *H, int32_t *argmax)
{
    if (M < 0 || V < 1 || K < 1)
        return -1;
    for (int m = 0; m < M; m++) {
        double *row = logits ? logits + (long long)m * V : (double *)malloc(sizeof(double) * (size_t)V);
        if (!row)
            return -1;
#pragma omp parallel for schedule(static)
        for (long long v = 0; v < V; v++) {
            double acc = 0.0;
            for (int k = 0; k < K; k++)
                acc += (double)half_to_float(x[(long long)m * K + k]) * (double)half_to_float(w[v * K + k]);
            row[v] = acc;
        }
        double mx = -INFINITY;
        int best = 0;
        for (int v = 0; v < V; v++)
            if (row[v] > mx) {
                mx = row[v];
                best = v;
            }
        double S = 0.0;
        for (int v = 0; v < V; v++)
            S += exp(row[v] - mx);
        const double lse = mx + log(S);
        double h = 0.0;
        for (int v = 0; v < V; v++) {
            double p = exp(row[v] - mx) / S;
            if (p != 0.0)
                h -= p * (row[v] - lse);
        }
        H[m] = h;
        if (argmax)
            argmax[m] = best;
        if (!logits)
            free(row);
    }
    return 0;
}

/* ---- Offline replacement order, Sec. 4.3 -------------------------------------------
 *
 * Linear layers with the smaller KL divergence are replaced first.  values: [n][m]
 * float, the KL of entry e on each of m calibration rows; the key of an entry is the sum
 * of its m values in double, taken in index order.  order[i] = the entry with the i-th
 * smallest key; equal keys keep their index order; keys that are NaN come last (again in
 * index order).  Plain insertion sort.
 */
int orc_rank_ascending(const float *values, int n, int m, int32_t *order)
{
    if (n < 0 || m < 1)
        return -1;
    for (int e = 0; e < n; e++) {
        double key = 0.0;
        for (int j = 0; j < m; j++)
            key += (double)values[(long long)e * m + j];
        /* insert e after every entry already placed whose key is <= key */
        int pos = e;
        while (pos > 0) {
            int prev = order[pos - 1];
            double pk = 0.0;
            for (int j = 0; j < m; j++)
                pk += (double)values[(long long)prev * m + j];
            int prev_after = isnan(pk) ? !isnan(key) : (!isnan(key) && pk > key);
            if (!prev_after)
                break;
            order[pos] = prev;
            pos--;
        }
        order[pos] = e;
    }
    return 0;
}

/* ---- W8A8 prefill, Sec. 4.1 / 4.3 / 4.5 ----------------------------------------------
 *
 * The prefill runs 8-bit weights against 8-bit activations on the integer matrix units.
 * The weights are the resident INT8 copy of orc_quantize.  The paper does not say how the
 * activations are quantized; the reading taken is the symmetric simplification stated
 * after Eq. (3), per token (row of x): z = 0, Xmax = -Xmin = max |x|,
 * q_max - q_min = 2^8 - 2, so s = (2 max|x|) / 254 and q = round(x / s) in [-127, 127],
 * in binary32 with one rounding per operation, round-half-to-even; an all-zero row gets
 * s = 1.  Returns -1 on a non-finite activation.
 */
int orc_quantize_act(const uint16_t *x, int M, int K, int8_t *xq, float *sx)
{
    if (M < 0 || K < 1)
        return -1;
    int bad = 0;
    for (long long m = 0; m < M; m++) {
        float amax = 0.0f;
        for (int k = 0; k < K; k++) {
            float v = fabsf(half_to_float(x[m * K + k]));
            if (!isfinite(v))
                bad = 1;
            if (v > amax) amax = v;
        }
        float s = 1.0f;
        if (amax > 0.0f) {
            volatile float range = amax + amax; /* Xmax - Xmin */
            volatile float sv = range / 254.0f;
            s = sv;
        }
        sx[m] = s;
        for (int k = 0; k < K; k++) {
            volatile float t = half_to_float(x[m * K + k]) / s;
            float q = rintf(t);
            if (q < -127.0f) q = -127.0f;
            if (q > 127.0f) q = 127.0f;
            xq[m * K + k] = (int8_t)q;
        }
    }
    return bad ? -1 : 0;
}

/*
 * y = x_hat . w_hat^T with both operands dequantized by Eq. (3): x_hat[m][k] =
 * xq[m][k] * sx[m] (z = 0) and w_hat as in orc_linear at 8 bits, each a binary32 value;
 * the sum over k runs in index order in double and is rounded once to binary16.
 * Rows row0 .. row0+rows-1 of the output; y: [M][rows].
 */
int orc_linear_w8a8(const int8_t *xq, const float *sx, int M, const uint8_t *codes,
                    const float *scales, const uint8_t *zeros, int N, int K, int group,
                    int row0, int rows, uint16_t *y)
{
    if (group <= 0 || K % group != 0 || row0 < 0 || rows < 0 || row0 + rows > N)
        return -1;
    const int G = K / group;
#pragma omp parallel for schedule(static)
    for (long long r = 0; r < rows; r++) {
        long long n = row0 + r;
        for (int m = 0; m < M; m++) {
            double acc = 0.0;
            for (long long k = 0; k < K; k++) {
                int g = (int)(k / group);
                volatile float d = (float)codes[n * K + k] - (float)zeros[n * G + g];
                volatile float wv = d * scales[n * G + g];
                volatile float xv = (float)xq[(long long)m * K + k] * sx[m];
                acc += (double)xv * (double)wv;
            }
            y[(long long)m * rows + r] = double_to_half(acc);
        }
    }
    return 0;
}
