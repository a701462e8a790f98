/*
 * CPU oracle for absorbed multi-head latent attention (MLA) decode over a
 * paged, compressed KV cache.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It defines what "correct" means for the
 * GPU library and is never linked into, imported by, or called from the
 * product path.  It shares no code with the HIP kernels.  Everything is plain
 * loops in fp64 on the exactly-widened stored values; nothing is blocked,
 * fused or reordered beyond what the cited equations state.
 *
 * Notation follows the paper (Sec. 3.3): h query heads (H), head dim d
 * (d_head), latent rank r_kv (d_c), decoupled-RoPE dim d^R (d_rope),
 * c_t^{KV} (c_kv), k_t^R (k_rope), q^C (q_nope), q^R (q_rope).
 * Row-vector storage: W_UK[h] is W^{UK}_h stored [d_head x d_c];
 * W_UV[h] is (W^{UV}_h)^T stored [d_c x d_head].
 *
 * Cache layout (paging is not in the paper; it is the serving layout this
 * oracle shares with the GPU library as an *interface*): a pool of
 * [num_pages][page_size] rows, each row = [c_kv (d_c) | k_rope (d_rope)].
 * Logical token j of sequence b lives in physical page
 * page_table[b*max_pages_per_seq + j/page_size], slot j%page_size.
 *
 * Cache dtypes: 0 = fp32, 1 = bf16 (uint16 bit patterns), 2 = OCP fp8 e4m3
 * codes with one fp32 scale per token (value = decode(code) * scale).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_FP8_E4M3 = 2 };

/* ---- exact widening of stored values ----------------------------------- */

/* bfloat16 is the upper 16 bits of an IEEE binary32. */
static double widen_bf16(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* OCP 8-bit float E4M3: 1 sign, 4 exponent (bias 7), 3 mantissa bits.
 * exponent 0 -> subnormal mant * 2^-9; S.1111.111 -> NaN; no infinities;
 * largest finite 1.75 * 2^8 = 448. */
static double widen_e4m3(uint8_t code)
{
    int sign = code >> 7, e = (code >> 3) & 0xF, m = code & 0x7;
    double v;
    if (e == 0xF && m == 0x7) return NAN;
    if (e == 0) v = ldexp((double)m, -9);
    else        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

double oracle_widen_bf16(uint16_t bits) { return widen_bf16(bits); }
double oracle_widen_e4m3(uint8_t code)  { return widen_e4m3(code); }

static size_t elem_bytes(int dtype)
{
    return dtype == ORC_F32 ? 4 : dtype == ORC_BF16 ? 2 : 1;
}

/* Widen one stored cache row (row_len values) to fp64. */
static void widen_row(const void* pool, const float* kv_scale, int dtype,
                      size_t row_index, int row_len, double* dst)
{
    size_t off = row_index * (size_t)row_len;
    if (dtype == ORC_F32) {
        const float* p = (const float*)pool + off;
        for (int i = 0; i < row_len; ++i) dst[i] = (double)p[i];
    } else if (dtype == ORC_BF16) {
        const uint16_t* p = (const uint16_t*)pool + off;
        for (int i = 0; i < row_len; ++i) dst[i] = widen_bf16(p[i]);
    } else {
        const uint8_t* p = (const uint8_t*)pool + off;
        double s = (double)kv_scale[row_index];
        for (int i = 0; i < row_len; ++i) dst[i] = widen_e4m3(p[i]) * s;
    }
}

/* Physical row index of logical token j of sequence b. */
static size_t phys_row(const int32_t* page_table, int max_pages_per_seq,
                       int page_size, int b, int j)
{
    int32_t page = page_table[(size_t)b * max_pages_per_seq + j / page_size];
    return (size_t)page * page_size + (size_t)(j % page_size);
}

/* Threads the (b, h) loops may use from now on (n >= 1); 0 restores the default. */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    static int dflt = 0;
    if (dflt == 0) dflt = omp_get_max_threads();
    omp_set_num_threads(n > 0 ? n : dflt);
#else
    (void)n;
#endif
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- page gather (byte-exact) ------------------------------------------ */

/* dense[b][j][:] = row bytes of logical token j, for j < seq_lens[b];
 * bytes of rows j >= seq_lens[b] are set to zero. */
int oracle_gather_paged(const void* pool, const int32_t* page_table,
                        const int32_t* seq_lens, void* dense, int B,
                        int max_len, int row_bytes, int page_size,
                        int max_pages_per_seq)
{
    const uint8_t* src = (const uint8_t*)pool;
    uint8_t* dst = (uint8_t*)dense;
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < max_len; ++j) {
            uint8_t* d = dst + ((size_t)b * max_len + j) * row_bytes;
            if (j < seq_lens[b]) {
                size_t r = phys_row(page_table, max_pages_per_seq, page_size, b, j);
                memcpy(d, src + r * row_bytes, (size_t)row_bytes);
            } else {
                memset(d, 0, (size_t)row_bytes);
            }
        }
    return 0;
}

/* ---- the two per-head projections (Eq. "mqa", first and last line) ----- */

/* q_abs[b,h,:] = (W^{UK}_h)^T q^C_{b,h}  ==  q_nope[b,h,:] . W_UK[h] */
int oracle_absorb_q(const double* q_nope, const double* W_UK, double* q_abs,
                    int B, int H, int d_head, int d_c)
{
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            const double* q = q_nope + ((size_t)b * H + h) * d_head;
            const double* W = W_UK + (size_t)h * d_head * d_c;
            double* o = q_abs + ((size_t)b * H + h) * d_c;
            for (int c = 0; c < d_c; ++c) {
                double acc = 0.0;
                for (int d = 0; d < d_head; ++d) acc += q[d] * W[(size_t)d * d_c + c];
                o[c] = acc;
            }
        }
    return 0;
}

/* out[b,h,:] = W^{UV}_h o_hat_{b,h}  ==  o_lat[b,h,:] . W_UV[h] */
int oracle_out_proj(const double* o_lat, const double* W_UV, double* out,
                    int B, int H, int d_c, int d_head)
{
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            const double* o = o_lat + ((size_t)b * H + h) * d_c;
            const double* W = W_UV + (size_t)h * d_c * d_head;
            double* y = out + ((size_t)b * H + h) * d_head;
            for (int d = 0; d < d_head; ++d) {
                double acc = 0.0;
                for (int c = 0; c < d_c; ++c) acc += o[c] * W[(size_t)c * d_head + d];
                y[d] = acc;
            }
        }
    return 0;
}

/* ---- softmax over one score vector, two passes, fp64 ------------------- */

/* In place: s[0..n) -> p[0..n); returns lse = m + log(sum exp(s - m)).
 * n == 0 returns -inf. */
static double softmax_inplace(double* s, int n)
{
    if (n == 0) return -INFINITY;
    double m = s[0];
    for (int j = 1; j < n; ++j) if (s[j] > m) m = s[j];
    double z = 0.0;
    for (int j = 0; j < n; ++j) { s[j] = exp(s[j] - m); z += s[j]; }
    for (int j = 0; j < n; ++j) s[j] /= z;
    return m + log(z);
}

/* ---- explicit ("MHA paradigm", Eq. "mha") form: the definition --------- */

/* For each selected (b,h): materialise k_j = [W^{UK}_h c_j ; k^R_j] and
 * v_j = W^{UV}_h c_j, score q = [q^C ; q^R] against k_j with the given
 * scale, softmax over j = 0..L-1, out = sum_j p_j v_j.
 * b_sel/h_sel (may be NULL = all) list the sequences / heads to compute;
 * outputs are indexed [ib][ih] over the selections.
 * probs (may be NULL): [n_b][n_h][max_len] softmax rows, zero padded. */
int oracle_decode_explicit(const double* q_nope, const double* q_rope,
                           const double* W_UK, const double* W_UV,
                           const void* pool, const float* kv_scale,
                           const int32_t* page_table, const int32_t* seq_lens,
                           double* out, double* lse, double* probs, int max_len,
                           int B, int H, int d_head, int d_c, int d_rope,
                           int page_size, int max_pages_per_seq,
                           double softmax_scale, int cache_dtype,
                           const int32_t* b_sel, int n_b,
                           const int32_t* h_sel, int n_h)
{
    (void)B;
    int row_len = d_c + d_rope;
    if (!b_sel) n_b = B;
    if (!h_sel) n_h = H;
    int n_task = n_b * n_h;
#pragma omp parallel for schedule(dynamic, 1)
    for (int task = 0; task < n_task; ++task) {
        int ib = task / n_h, ih = task % n_h;
        int b = b_sel ? b_sel[ib] : ib;
        int h = h_sel ? h_sel[ih] : ih;
        int L = seq_lens[b];
        const double* qc = q_nope + ((size_t)b * H + h) * d_head;
        const double* qr = q_rope + ((size_t)b * H + h) * d_rope;
        const double* Wk = W_UK + (size_t)h * d_head * d_c;
        const double* Wv = W_UV + (size_t)h * d_c * d_head;
        double* row = (double*)malloc(sizeof(double) * row_len);
        double* s   = (double*)malloc(sizeof(double) * (L > 0 ? L : 1));
        double* V   = (double*)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1) * d_head);
        double* kc  = (double*)malloc(sizeof(double) * d_head);
        for (int j = 0; j < L; ++j) {
            size_t r = phys_row(page_table, max_pages_per_seq, page_size, b, j);
            widen_row(pool, kv_scale, cache_dtype, r, row_len, row);
            /* k^C_{j,h} = W^{UK}_h c_j */
            for (int d = 0; d < d_head; ++d) {
                double acc = 0.0;
                for (int c = 0; c < d_c; ++c) acc += Wk[(size_t)d * d_c + c] * row[c];
                kc[d] = acc;
            }
            /* v_{j,h} = W^{UV}_h c_j */
            for (int d = 0; d < d_head; ++d) {
                double acc = 0.0;
                for (int c = 0; c < d_c; ++c) acc += row[c] * Wv[(size_t)c * d_head + d];
                V[(size_t)j * d_head + d] = acc;
            }
            double dot = 0.0;
            for (int d = 0; d < d_head; ++d) dot += qc[d] * kc[d];
            for (int r2 = 0; r2 < d_rope; ++r2) dot += qr[r2] * row[d_c + r2];
            s[j] = softmax_scale * dot;
        }
        double l = softmax_inplace(s, L);
        double* o = out + ((size_t)ib * n_h + ih) * d_head;
        for (int d = 0; d < d_head; ++d) o[d] = 0.0;
        for (int j = 0; j < L; ++j)
            for (int d = 0; d < d_head; ++d) o[d] += s[j] * V[(size_t)j * d_head + d];
        if (lse) lse[(size_t)ib * n_h + ih] = l;
        if (probs) {
            double* pr = probs + ((size_t)ib * n_h + ih) * max_len;
            for (int j = 0; j < max_len; ++j) pr[j] = j < L ? s[j] : 0.0;
        }
        free(row); free(s); free(V); free(kc);
    }
    return 0;
}

/* ---- absorbed ("MQA paradigm", Eq. "mqa") form -------------------------- */

/* Core for one (b,h) over logical tokens [j0, j1): q_hat = [q_abs ; q_rope],
 * k_hat_j = [c_j ; k^R_j]; s_j = scale * q_hat . k_hat_j; p = softmax;
 * o_hat = sum_j p_j c_j.  Returns lse (-inf and o_hat = 0 if empty). */
static double absorbed_range(const double* qa, const double* qr,
                             const void* pool, const float* kv_scale,
                             const int32_t* page_table, int b, int j0, int j1,
                             double* o_hat, int d_c, int d_rope, int page_size,
                             int max_pages_per_seq, double softmax_scale,
                             int cache_dtype)
{
    int n = j1 > j0 ? j1 - j0 : 0;
    int row_len = d_c + d_rope;
    for (int c = 0; c < d_c; ++c) o_hat[c] = 0.0;
    if (n == 0) return -INFINITY;
    double* row = (double*)malloc(sizeof(double) * row_len);
    double* s   = (double*)malloc(sizeof(double) * n);
    for (int j = j0; j < j1; ++j) {
        size_t r = phys_row(page_table, max_pages_per_seq, page_size, b, j);
        widen_row(pool, kv_scale, cache_dtype, r, row_len, row);
        double dot = 0.0;
        for (int c = 0; c < d_c; ++c) dot += qa[c] * row[c];
        for (int r2 = 0; r2 < d_rope; ++r2) dot += qr[r2] * row[d_c + r2];
        s[j - j0] = softmax_scale * dot;
    }
    double l = softmax_inplace(s, n);
    for (int j = j0; j < j1; ++j) {
        size_t r = phys_row(page_table, max_pages_per_seq, page_size, b, j);
        widen_row(pool, kv_scale, cache_dtype, r, row_len, row);
        double p = s[j - j0];
        for (int c = 0; c < d_c; ++c) o_hat[c] += p * row[c];
    }
    free(row); free(s);
    return l;
}

/* o_lat[b,h,:] and lse[b,h] for every (b,h).  Threads (OpenMP) run over
 * (b,h); each (b,h) is computed exactly as written above. */
int oracle_decode_absorbed(const double* q_abs, const double* q_rope,
                           const void* pool, const float* kv_scale,
                           const int32_t* page_table, const int32_t* seq_lens,
                           double* o_lat, double* lse,
                           int B, int H, int d_c, int d_rope, int page_size,
                           int max_pages_per_seq, double softmax_scale,
                           int cache_dtype)
{
    int n_task = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int task = 0; task < n_task; ++task) {
        int b = task / H;
        double l = absorbed_range(q_abs + (size_t)task * d_c,
                                  q_rope + (size_t)task * d_rope,
                                  pool, kv_scale, page_table, b, 0, seq_lens[b],
                                  o_lat + (size_t)task * d_c, d_c, d_rope,
                                  page_size, max_pages_per_seq, softmax_scale,
                                  cache_dtype);
        if (lse) lse[task] = l;
    }
    return 0;
}

/* ---- several query tokens per sequence (multi-token prediction, speculative
 * decoding: the abstract's "Multi-Token Prediction"; Eq. "mqa" read for the T
 * newest positions at once) ------------------------------------------------
 * The cache of sequence b holds L = seq_lens[b] rows, the last T of which
 * belong to the T query tokens themselves.  Query token i (0 <= i < T) sits at
 * position t_i = L - T + i (0-based) and, by the sum over j = 1..t of
 * Eq. "mqa", attends to the cached rows 0 .. t_i, i.e. to the first
 * L - (T - 1 - i) rows.  A query token whose position is negative (L < T)
 * attends to nothing: o_hat = 0, lse = -inf.
 * q_abs [B,T,H,d_c], q_rope [B,T,H,d_rope] -> o_lat [B,T,H,d_c], lse [B,T,H]. */
int oracle_decode_absorbed_multi(const double* q_abs, const double* q_rope,
                                 const void* pool, const float* kv_scale,
                                 const int32_t* page_table, const int32_t* seq_lens,
                                 double* o_lat, double* lse,
                                 int B, int T, int H, int d_c, int d_rope,
                                 int page_size, int max_pages_per_seq,
                                 double softmax_scale, int cache_dtype)
{
    int n_task = B * T * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int task = 0; task < n_task; ++task) {
        int b = task / (T * H);
        int i = (task / H) % T;
        int visible = seq_lens[b] - (T - 1 - i);   /* rows 0 .. t_i */
        if (visible < 0) visible = 0;
        double l = absorbed_range(q_abs + (size_t)task * d_c,
                                  q_rope + (size_t)task * d_rope,
                                  pool, kv_scale, page_table, b, 0, visible,
                                  o_lat + (size_t)task * d_c, d_c, d_rope,
                                  page_size, max_pages_per_seq, softmax_scale,
                                  cache_dtype);
        if (lse) lse[task] = l;
    }
    return 0;
}

/* ---- prefill in the "MHA paradigm" (Eq. "mha"; Sec. 3.3 names it the form for
 * the compute-intensive phase): keys and values are materialised per head,
 *     k_{j,h} = [W^{UK}_h c_j ; k^R_j],    v_{j,h} = W^{UV}_h c_j,
 * and query token i of T (position t_i = L - T + i, as in the multi-token
 * decode above) attends to j = 0 .. t_i:
 *     o_{i,h} = sum_{j <= t_i} softmax_j( q_{i,h} . k_{j,h} * scale ) v_{j,h}.
 * T = L is the prefill of a whole prompt, T < L a later chunk of it.
 * q_nope [B,T,H,d_head], q_rope [B,T,H,d_rope] -> out [B,T,H,d_head], lse [B,T,H].
 * Threads run over (b,h); keys and values of one (b,h) are built once. */
int oracle_prefill_explicit(const double* q_nope, const double* q_rope,
                            const double* W_UK, const double* W_UV,
                            const void* pool, const float* kv_scale,
                            const int32_t* page_table, const int32_t* seq_lens,
                            double* out, double* lse,
                            int B, int T, int H, int d_head, int d_c, int d_rope,
                            int page_size, int max_pages_per_seq,
                            double softmax_scale, int cache_dtype)
{
    int row_len = d_c + d_rope;
    int dk = d_head + d_rope;
    int n_task = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int task = 0; task < n_task; ++task) {
        int b = task / H, h = task % H;
        int L = seq_lens[b];
        if (L < 0) L = 0;
        const double* Wk = W_UK + (size_t)h * d_head * d_c;
        const double* Wv = W_UV + (size_t)h * d_c * d_head;
        size_t n = (size_t)(L > 0 ? L : 1);
        double* row = (double*)malloc(sizeof(double) * row_len);
        double* K   = (double*)malloc(sizeof(double) * n * dk);
        double* V   = (double*)malloc(sizeof(double) * n * d_head);
        double* s   = (double*)malloc(sizeof(double) * n);
        for (int j = 0; j < L; ++j) {
            size_t r = phys_row(page_table, max_pages_per_seq, page_size, b, j);
            widen_row(pool, kv_scale, cache_dtype, r, row_len, row);
            for (int d = 0; d < d_head; ++d) {          /* k^C_{j,h} = W^{UK}_h c_j */
                double acc = 0.0;
                for (int c = 0; c < d_c; ++c) acc += Wk[(size_t)d * d_c + c] * row[c];
                K[(size_t)j * dk + d] = acc;
            }
            for (int r2 = 0; r2 < d_rope; ++r2) K[(size_t)j * dk + d_head + r2] = row[d_c + r2];
            for (int d = 0; d < d_head; ++d) {          /* v_{j,h} = W^{UV}_h c_j */
                double acc = 0.0;
                for (int c = 0; c < d_c; ++c) acc += row[c] * Wv[(size_t)c * d_head + d];
                V[(size_t)j * d_head + d] = acc;
            }
        }
        for (int i = 0; i < T; ++i) {
            size_t qi = ((size_t)b * T + i) * H + h;
            const double* qc = q_nope + qi * d_head;
            const double* qr = q_rope + qi * d_rope;
            int visible = L - (T - 1 - i);               /* keys 0 .. t_i */
            if (visible < 0) visible = 0;
            for (int j = 0; j < visible; ++j) {
                double dot = 0.0;
                for (int d = 0; d < d_head; ++d) dot += qc[d] * K[(size_t)j * dk + d];
                for (int r2 = 0; r2 < d_rope; ++r2) dot += qr[r2] * K[(size_t)j * dk + d_head + r2];
                s[j] = softmax_scale * dot;
            }
            double l = softmax_inplace(s, visible);
            double* o = out + qi * d_head;
            for (int d = 0; d < d_head; ++d) o[d] = 0.0;
            for (int j = 0; j < visible; ++j)
                for (int d = 0; d < d_head; ++d) o[d] += s[j] * V[(size_t)j * d_head + d];
            if (lse) lse[qi] = l;
        }
        free(row); free(K); free(V); free(s);
    }
    return 0;
}

/* ---- split-KV: chunk-local softmax, then log-sum-exp merge ------------- */

/* lse = log sum_s exp(lse_s); o = sum_s exp(lse_s - lse) o_s.
 * Chunks with lse_s = -inf carry weight 0; all empty -> o = 0, lse = -inf. */
int oracle_merge_lse(const double* o_part, const double* lse_part, int n_splits,
                     int d_c, double* o, double* lse_out)
{
    double m = -INFINITY;
    for (int s = 0; s < n_splits; ++s) if (lse_part[s] > m) m = lse_part[s];
    for (int c = 0; c < d_c; ++c) o[c] = 0.0;
    if (m == -INFINITY) { *lse_out = -INFINITY; return 0; }
    double z = 0.0;
    for (int s = 0; s < n_splits; ++s)
        if (lse_part[s] != -INFINITY) z += exp(lse_part[s] - m);
    double l = m + log(z);
    for (int s = 0; s < n_splits; ++s) {
        if (lse_part[s] == -INFINITY) continue;
        double w = exp(lse_part[s] - l);
        for (int c = 0; c < d_c; ++c) o[c] += w * o_part[(size_t)s * d_c + c];
    }
    *lse_out = l;
    return 0;
}

/* Sequence b's pages [0, ceil(L/page_size)) are cut into n_splits contiguous
 * chunks of chunk_pages pages each (the last ones may be short or empty);
 * each chunk gets its own softmax and (o_s, lse_s); the chunks are merged.
 * o_part [B,H,n_splits,d_c] and lse_part [B,H,n_splits] may be NULL. */
int oracle_decode_split(const double* q_abs, const double* q_rope,
                        const void* pool, const float* kv_scale,
                        const int32_t* page_table, const int32_t* seq_lens,
                        double* o_lat, double* lse,
                        double* o_part, double* lse_part,
                        int B, int H, int d_c, int d_rope, int page_size,
                        int max_pages_per_seq, int n_splits, int chunk_pages,
                        double softmax_scale, int cache_dtype)
{
    int n_task = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int task = 0; task < n_task; ++task) {
        int b = task / H;
        int L = seq_lens[b];
        double* op = (double*)malloc(sizeof(double) * (size_t)n_splits * d_c);
        double* lp = (double*)malloc(sizeof(double) * n_splits);
        for (int s = 0; s < n_splits; ++s) {
            long j0 = (long)s * chunk_pages * page_size;
            long j1 = j0 + (long)chunk_pages * page_size;
            if (j0 > L) j0 = L;
            if (j1 > L) j1 = L;
            lp[s] = absorbed_range(q_abs + (size_t)task * d_c,
                                   q_rope + (size_t)task * d_rope,
                                   pool, kv_scale, page_table, b, (int)j0, (int)j1,
                                   op + (size_t)s * d_c, d_c, d_rope, page_size,
                                   max_pages_per_seq, softmax_scale, cache_dtype);
        }
        double l;
        oracle_merge_lse(op, lp, n_splits, d_c, o_lat + (size_t)task * d_c, &l);
        if (lse) lse[task] = l;
        if (o_part) memcpy(o_part + (size_t)task * n_splits * d_c, op,
                           sizeof(double) * (size_t)n_splits * d_c);
        if (lse_part) memcpy(lse_part + (size_t)task * n_splits, lp,
                             sizeof(double) * n_splits);
        free(op); free(lp);
    }
    return 0;
}

/* ======================================================================
 * Cache append: the step that produces the row the decode reads.
 * Sec. 3.3 (MLA equations, left column):
 *     c_t^{KV} = W^{DKV} x_t          k_t^R = RoPE(W^{KR} x_t, t)
 * and the row kept per token is their concatenation [c^{KV} ; k^R]
 * (App. D.2: the r_kv-dimensional latent is what the cache stores).
 * RoPE is Sec. 3.1, Eq. 1: consecutive pairs (real, imaginary), pair i
 * rotated by the angle t * base^(-2i/d).
 * Storage encoders take their rounding decision on the fp32 value, the
 * precision the GPU library holds the row in before it stores it.
 * ====================================================================== */

/* row[j] = sum_k x[k] W[k][j] : W is [D][n], column j of it is row j of
 * the stacked matrix (W^{DKV} ; W^{KR}) (row-vector storage). */
int oracle_kv_row(const double* x, const double* W, int D, int n, double* row)
{
    for (int j = 0; j < n; ++j) {
        double acc = 0.0;
        for (int k = 0; k < D; ++k) acc += x[k] * W[(size_t)k * n + j];
        row[j] = acc;
    }
    return 0;
}

/* Eq. 1 on a vector of even length d at position pos, in place. */
int oracle_rope(double* v, int d, double pos, double base)
{
    if (d % 2) return -1;
    for (int i = 0; i < d / 2; ++i) {
        double theta = pow(base, -2.0 * (double)i / (double)d);
        double c = cos(pos * theta), s = sin(pos * theta);
        double re = v[2 * i], im = v[2 * i + 1];
        v[2 * i]     = re * c - im * s;
        v[2 * i + 1] = re * s + im * c;
    }
    return 0;
}

/* fp32 -> bfloat16 bits, round to nearest, ties to even (NaN kept quiet). */
uint16_t oracle_encode_bf16(float f)
{
    if (f != f) return 0x7FC0;
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    uint32_t lo = u & 0xFFFFu, hi = u >> 16;
    if (lo > 0x8000u || (lo == 0x8000u && (hi & 1u))) hi += 1;  /* carries into the exponent as it must */
    return (uint16_t)hi;
}

/* fp32 -> OCP e4m3 code: the nearest representable value, ties to the code
 * with even mantissa, magnitudes beyond 448 saturate to 448 (the format has
 * no infinity).  Brute force over the 254 finite codes. */
uint8_t oracle_encode_e4m3(float f)
{
    if (f != f) return 0x7F;
    double a = fabs((double)f);
    int best = 0;
    double best_err = INFINITY;
    for (int c = 0; c < 0x7F; ++c) {          /* positive codes, 0x7F is NaN */
        double err = fabs(widen_e4m3((uint8_t)c) - a);
        if (err < best_err || (err == best_err && (c & 1) == 0)) { best = c; best_err = err; }
    }
    return (uint8_t)(best | (signbit(f) ? 0x80 : 0));
}

/* One token's row in fp32 -> storage.  fp8: one scale per token over the
 * whole row, scale = absmax/448 (1 for an all-zero row), code =
 * encode(value/scale), both divisions in fp32. */
int oracle_encode_row(const float* row, int n, int dtype, void* dst, float* scale_out)
{
    if (dtype == ORC_F32) {
        memcpy(dst, row, (size_t)n * 4);
    } else if (dtype == ORC_BF16) {
        for (int j = 0; j < n; ++j) ((uint16_t*)dst)[j] = oracle_encode_bf16(row[j]);
    } else {
        float amax = 0.f;
        for (int j = 0; j < n; ++j) { float a = fabsf(row[j]); if (a > amax) amax = a; }
        float scale = amax > 0.f ? amax / 448.0f : 1.0f;
        for (int j = 0; j < n; ++j) ((uint8_t*)dst)[j] = oracle_encode_e4m3(row[j] / scale);
        if (scale_out) *scale_out = scale;
    }
    return 0;
}

/* For every sequence b: row = [W^{DKV} x_b ; RoPE(W^{KR} x_b, pos_b)] written
 * to logical position pos_b of that sequence (page page_table[b][pos_b /
 * page_size], slot pos_b % page_size).  x [B][D], W [D][d_c + d_rope] fp64
 * (already widened); rows_out (optional) receives the fp64 rows.  A
 * position outside the table, or a page id outside the pool, leaves that
 * sequence untouched. */
int oracle_cache_append(const double* x, const double* W, void* pool, float* kv_scale,
                        int dtype, const int32_t* page_table, const int32_t* positions,
                        int B, int D, int d_c, int d_rope, int page_size, int num_pages,
                        int max_pages_per_seq, double rope_base, double* rows_out)
{
    const int n = d_c + d_rope;
    double* row = (double*)malloc((size_t)n * sizeof(double));
    float* row32 = (float*)malloc((size_t)n * sizeof(float));
    if (!row || !row32) { free(row); free(row32); return -1; }
    for (int b = 0; b < B; ++b) {
        oracle_kv_row(x + (size_t)b * D, W, D, n, row);
        oracle_rope(row + d_c, d_rope, (double)positions[b], rope_base);
        if (rows_out) memcpy(rows_out + (size_t)b * n, row, (size_t)n * sizeof(double));
        int pos = positions[b];
        if (pos < 0 || pos >= max_pages_per_seq * page_size) continue;
        int32_t page = page_table[(size_t)b * max_pages_per_seq + pos / page_size];
        if (page < 0 || page >= num_pages) continue;
        size_t r = (size_t)page * page_size + (size_t)(pos % page_size);
        for (int j = 0; j < n; ++j) row32[j] = (float)row[j];
        oracle_encode_row(row32, n, dtype, (uint8_t*)pool + r * n * elem_bytes(dtype),
                          kv_scale ? kv_scale + r : NULL);
    }
    free(row);
    free(row32);
    return 0;
}

size_t oracle_elem_bytes(int dtype) { return elem_bytes(dtype); }
