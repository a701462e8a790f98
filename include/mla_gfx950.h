/*
 * mla_gfx950.h -- C ABI of the absorbed multi-head latent attention (MLA)
 * decode library for AMD MI355X (gfx950).
 *
 * The three main compute calls are the three lines of the paper's absorbed
 * ("MQA paradigm") attention equation in Sec. 3.3:
 *
 *   q_hat_i = [ (W^{UK}_i)^T q^C_i ; q^R_i ]                    mla_absorb_q
 *   o_hat_i = sum_j softmax_j( q_hat_i . k_hat_j * scale ) c_j  mla_decode_paged
 *             with k_hat_j = [ c_j^{KV} ; k_j^R ]
 *   o_i     = W^{UV}_i o_hat_i                                  mla_out_proj
 *
 * Notation: H query heads (paper: h), d_head (d), latent rank d_c (r_kv),
 * decoupled-RoPE width d_rope (d^R).  The final W^O projection and the
 * projections that produce q^C and q^R are outside this library.
 * q_rope and the k_rope part of the cache are passed ALREADY rotated by RoPE
 * to the three calls above; mla_cache_append is the one call that produces a
 * cache row (c^{KV} and the rotated k^R of a new token) and applies RoPE.
 *
 * General conventions
 *  - Every pointer is a DEVICE pointer unless the comment says "host".
 *    The caller owns every buffer, including the workspace; the library
 *    allocates no device memory.  It keeps no state between calls that a
 *    result depends on; what it does keep per process is bookkeeping: which
 *    kernels have had their dynamic-LDS limit raised (conversion kernels),
 *    and, per device, the address of the static scratch array of
 *    mla_decode_paged_static.
 *  - Tensors are dense, row-major, innermost index last, and 16-byte aligned.
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *    All work is enqueued on it and the call returns without waiting.
 *  - Return value: MLA_OK (0) or a negative mla_status.  Arguments are
 *    validated on the host before the first HIP call; on error nothing is
 *    launched and no output is written.  Nothing throws across this ABI.
 *  - "io dtype" is the type of q / weights / outputs (MLA_F32 or MLA_BF16);
 *    all accumulation is fp32.
 */
#ifndef MLA_GFX950_H
#define MLA_GFX950_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MLA_F32      = 0,  /* IEEE binary32                                        */
    MLA_BF16     = 1,  /* bfloat16 (upper half of binary32)                    */
    MLA_FP8_E4M3 = 2   /* OCP E4M3 (max 448, no inf); cache storage only       */
} mla_dtype;

typedef enum {
    MLA_OK              =  0,
    MLA_ERR_NULL        = -1,  /* a required pointer is NULL                   */
    MLA_ERR_SHAPE       = -2,  /* a size is <= 0 or inconsistent               */
    MLA_ERR_UNSUPPORTED = -3,  /* shape / dtype combination not implemented    */
    MLA_ERR_WORKSPACE   = -4,  /* workspace missing or too small               */
    MLA_ERR_HIP         = -6,  /* a HIP runtime call (launch) failed           */
    MLA_ERR_SCRATCH_LIMIT = -7 /* mla_decode_paged_static: the sizes need more
                                  scratch than the library's static array holds */
} mla_status;

/* Flags for mla_decode_paged. */
enum {
    MLA_FLAG_DEFAULT        = 0,
    MLA_FLAG_PORTABLE_KERNEL = 1, /* force the scalar-FMA kernel even where the
                                     matrix-core kernel applies (cross-check)  */
    MLA_FLAG_SKIP_MERGE      = 2, /* leave the per-chunk partial results in the
                                     workspace and do not write o_lat / lse: the
                                     caller merges them with mla_merge_partials
                                     (o_lat may then be NULL)                  */
    MLA_FLAG_BALANCED        = 4  /* balanced partition (see mla_decode_paged);
                                     the merge calls that consume the workspace
                                     must be given the same flag               */
};

/* Human-readable name of a status code.  Static storage; never free it. */
const char* mla_status_string(int status);

/* Library version as a static string. */
const char* mla_version(void);

/*
 * Absorb (first line of the absorbed equation; App. A.2.2 folds the same
 * product into W'^Q):   q_abs[b,h,:] = q_nope[b,h,:] . W_UK[h]
 *
 *   q_nope [B, H, d_head]    io dtype
 *   W_UK   [H, d_head, d_c]  io dtype; W_UK[h] is W^{UK}_h (rows = head dims)
 *   q_abs  [B, H, d_c]       io dtype (output)
 * Any B, H, d_head, d_c >= 1.
 */
int mla_absorb_q(const void* q_nope, const void* W_UK, void* q_abs,
                 int B, int H, int d_head, int d_c,
                 mla_dtype io_dtype, void* hip_stream);

/*
 * Output up-projection (last line of the absorbed equation, inside the
 * brackets):            out[b,h,:] = o_lat[b,h,:] . W_UV[h]
 *
 *   o_lat [B, H, d_c]        io dtype
 *   W_UV  [H, d_c, d_head]   io dtype; W_UV[h] is (W^{UV}_h)^T
 *   out   [B, H, d_head]     io dtype (output)
 */
int mla_out_proj(const void* o_lat, const void* W_UV, void* out,
                 int B, int H, int d_c, int d_head,
                 mla_dtype io_dtype, void* hip_stream);

/*
 * Bytes of device workspace mla_decode_paged needs for these sizes (split-KV
 * partial results for B * (S + 1) chunks, S as described under num_splits:
 * partial outputs in the io dtype, sized here as if they were fp32, and fp32
 * log-sum-exps; plus a [B, 2] int32 table the balanced partition uses).  The
 * same size serves both partitions and both io dtypes.  What the workspace
 * holds after MLA_FLAG_SKIP_MERGE is for the merge calls of this library only.
 * Pure host function; returns 0 if an argument is <= 0.
 */
size_t mla_decode_workspace_bytes(int B, int H, int d_c, int num_splits);

/*
 * Paged absorbed decode (second line of the absorbed equation).  For every
 * sequence b and head h, over the cached tokens j = 0 .. seq_lens[b]-1 (the
 * current token's row is already in the cache; no other mask):
 *
 *   s_j   = softmax_scale * ( q_abs[b,h,:] . c_kv[j] + q_rope[b,h,:] . k_rope[j] )
 *   p     = softmax_j(s)
 *   o_lat[b,h,:] = sum_j p_j c_kv[j]          lse[b,h] = log sum_j exp(s_j)
 *
 *   q_abs      [B, H, d_c]     io dtype
 *   q_rope     [B, H, d_rope]  io dtype, already rotated (position seq_len-1)
 *   kv_cache   [num_pages, page_size, d_c + d_rope]  cache dtype; one pool,
 *              row = [ c_kv | k_rope ], k_rope already rotated at its position
 *   kv_scale   [num_pages, page_size] fp32: required iff cache dtype is
 *              MLA_FP8_E4M3 (stored value = decode(code) * scale of that
 *              token); must be NULL otherwise
 *   page_table [B, max_pages_per_seq] int32: logical token j of sequence b
 *              is row (j % page_size) of page page_table[b][j / page_size].
 *              Entries at or beyond ceil(seq_len/page_size) are never read
 *              (they may be -1).  An entry outside [0, num_pages) that WOULD
 *              be read is not an error code (the table is device memory):
 *              the tokens of that page are skipped.
 *   seq_lens   [B] int32, each in [0, max_pages_per_seq * page_size].
 *              Slots of the last page past seq_len, and pages not in the
 *              table, are never used (they may hold NaN).
 *   o_lat      [B, H, d_c] io dtype (output);  seq_len 0 gives zeros
 *   lse        [B, H] fp32 natural-log-sum-exp of the scaled scores (output,
 *              may be NULL);  seq_len 0 gives -inf
 *   workspace  at least mla_decode_workspace_bytes(B, H, d_c, num_splits)
 *              bytes, 256-byte aligned; contents are scratch
 *   num_splits >= 1: each sequence's page list is cut into S contiguous
 *              chunks of ceil(max_pages_per_seq / S) pages (trailing chunks of
 *              short sequences are empty), S = num_splits, or 2x / 4x that
 *              while B * S stays below 256 (so a small batch still gives
 *              every compute unit a workgroup; mla_decode_workspace_bytes
 *              accounts for it).  Every chunk is reduced with its own running
 *              softmax and the chunks are merged by log-sum-exp.  The result
 *              does not depend on the chunking beyond fp32 rounding.
 *              With MLA_FLAG_BALANCED (matrix-core kernel only, otherwise
 *              MLA_ERR_UNSUPPORTED) the cut is made differently: the page lists
 *              of all sequences, laid end to end, are cut into B * S ranges of
 *              equal length (+-1 page), one per workgroup; a range that
 *              crosses sequence boundaries gives one chunk per sequence.  Every
 *              workgroup then streams the same number of bytes whatever the
 *              mix of sequence lengths.  Same results up to fp32 rounding.
 *   softmax_scale  the paper uses 1/sqrt(d_head + d_rope) for MLA
 *
 * Supported: io/cache dtype pairs (F32,F32), (BF16,BF16), (BF16,FP8_E4M3),
 * (F32,BF16), (F32,FP8_E4M3); 1 <= H <= 1024; d_c a multiple of 8 up to 512;
 * d_rope a multiple of 8 in [0, 64]; any page_size >= 1.
 * The matrix-core (MFMA) kernel is used for BF16 io with a BF16 or FP8 cache,
 * page_size 64, d_rope 64 and d_c in {256, 512} (32 heads per workgroup; more
 * heads go to further workgroups); everything else runs on the portable
 * scalar-FMA kernel.
 */
int mla_decode_paged(const void* q_abs, const void* q_rope,
                     const void* kv_cache, const float* kv_scale,
                     const int32_t* page_table, const int32_t* seq_lens,
                     void* o_lat, float* lse,
                     void* workspace, size_t workspace_bytes,
                     int B, int H, int d_c, int d_rope, int page_size,
                     int num_pages, int max_pages_per_seq, int num_splits,
                     float softmax_scale, mla_dtype io_dtype,
                     mla_dtype cache_dtype, unsigned flags, void* hip_stream);

/*
 * mla_decode_paged for callers that cannot allocate and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and kernels as mla_decode_paged,
 * without `workspace` / `workspace_bytes`: the split-KV partial results live
 * in a device array that is part of the library's code object
 * (mla_static_scratch_bytes() = 32 MiB; every GPU the library runs on holds its
 * own copy until the process ends).  The call allocates and frees nothing.
 *
 *  - Sizes for which mla_decode_workspace_bytes(B, H, d_c, num_splits) exceeds
 *    mla_static_scratch_bytes() are rejected with MLA_ERR_SCRATCH_LIMIT before
 *    anything is launched (the headline shape B 16, H 32, d_c 512, 16 chunks
 *    needs 17.9 MB).
 *  - MLA_FLAG_SKIP_MERGE is rejected (MLA_ERR_UNSUPPORTED): the partials would
 *    stay in an array the caller cannot name.  The other flags work as usual.
 *  - The device that owns the buffers and the stream must be the current
 *    device of the calling thread.  On its first call on a device the library
 *    looks up that device's address of the array (hipGetSymbolAddress; no
 *    allocation) and keeps it.
 *  - All calls on one GPU share that GPU's array, which keeps the previous
 *    call's contents; nothing in it needs clearing (every partial that is read
 *    has been written by the same call, or is discarded by a select).  Calls
 *    that overlap on one GPU (different streams, or several host threads) race
 *    on it: serialise them, or use mla_decode_paged with separate workspaces.
 */
size_t mla_static_scratch_bytes(void);
int mla_decode_paged_static(const void* q_abs, const void* q_rope,
                            const void* kv_cache, const float* kv_scale,
                            const int32_t* page_table, const int32_t* seq_lens,
                            void* o_lat, float* lse,
                            int B, int H, int d_c, int d_rope, int page_size,
                            int num_pages, int max_pages_per_seq, int num_splits,
                            float softmax_scale, mla_dtype io_dtype,
                            mla_dtype cache_dtype, unsigned flags, void* hip_stream);

/*
 * mla_decode_paged for q_len query tokens per sequence in one pass over the
 * cache (multi-token prediction / speculative decoding, which the paper's
 * abstract names as a further speed-up of the converted model; the second line
 * of the absorbed equation in Sec. 3.3 read for the q_len newest positions at
 * once).  The cache of sequence b already holds the rows of its q_len query
 * tokens: they are its last q_len rows.  Query token i (0 <= i < q_len) sits
 * at position seq_lens[b] - q_len + i and, as the sum over j = 1..t of that
 * equation says, sees the cached rows up to and including its own, i.e. the
 * first seq_lens[b] - (q_len - 1 - i) rows; a token whose position would be
 * negative sees nothing (zeros, lse = -inf).
 *
 *   q_abs   [B, q_len, heads, d_c]     q_rope [B, q_len, heads, d_rope]
 *   o_lat   [B, q_len, heads, d_c]     lse    [B, q_len, heads]
 *   workspace  sized by mla_decode_workspace_bytes(B, q_len * heads, d_c,
 *              num_splits); the same H = q_len * heads goes to
 *              mla_merge_partials.  mla_absorb_q and mla_out_proj take the
 *              query tokens as a batch of B * q_len.
 * Everything else as for mla_decode_paged, which is this call with q_len 1.
 * BF16 caches with the uniform partition: 64 query rows (e.g. two tokens of
 * 32 heads) share one pass over the cached rows; further groups of 64 rows run
 * beside the first on the same XCD and find the rows in its L2.  FP8 caches
 * and MLA_FLAG_BALANCED: groups of 32 query rows.  q_len * heads <= 1024.
 */
int mla_decode_paged_multi(const void* q_abs, const void* q_rope,
                           const void* kv_cache, const float* kv_scale,
                           const int32_t* page_table, const int32_t* seq_lens,
                           void* o_lat, float* lse,
                           void* workspace, size_t workspace_bytes,
                           int B, int q_len, int heads, int d_c, int d_rope,
                           int page_size, int num_pages, int max_pages_per_seq,
                           int num_splits, float softmax_scale,
                           mla_dtype io_dtype, mla_dtype cache_dtype,
                           unsigned flags, void* hip_stream);

/*
 * Split-KV reduction on its own: merges the per-chunk partial results a
 * mla_decode_paged call (same B, H, d_c, num_splits, same workspace) left
 * behind, exactly as that call does when MLA_FLAG_SKIP_MERGE is not set:
 *   lse = log sum_s exp(lse_s),   o_lat = sum_s exp(lse_s - lse) o_s
 * (chunks with lse_s = -inf are skipped; all empty gives zeros and -inf).
 * This is the softmax identity behind chunked evaluation; it lets a caller
 * time or overlap the two phases, or merge chunks computed elsewhere.
 *   workspace  [in]  as written by mla_decode_paged
 *   o_lat      [B, H, d_c] io dtype (output);  lse [B, H] fp32 (output, may be NULL)
 *   flags      MLA_FLAG_BALANCED iff the decode call had it; other bits ignored
 */
int mla_merge_partials(const void* workspace, size_t workspace_bytes,
                       void* o_lat, float* lse, int B, int H, int d_c,
                       int num_splits, mla_dtype io_dtype, unsigned flags,
                       void* hip_stream);

/*
 * Fused tail: mla_merge_partials followed by mla_out_proj in one call (one
 * kernel where the shapes allow: bf16 io, d_head 128, d_c 256 or 512, at most
 * 64 chunks of the uniform partition or any balanced one; otherwise the two
 * kernels back to back).  Same results as the two
 * calls: o_lat is the merged latent output rounded to the io dtype, and out is
 * computed from that rounded o_lat.
 *   workspace  [in]  as written by mla_decode_paged(..., MLA_FLAG_SKIP_MERGE)
 *   W_UV       [H, d_c, d_head] io dtype
 *   o_lat      [B, H, d_c] io dtype (output, required)
 *   lse        [B, H] fp32 (output, may be NULL)
 *   out        [B, H, d_head] io dtype (output)
 *   flags      MLA_FLAG_BALANCED iff the decode call had it; other bits ignored
 */
int mla_merge_out_proj(const void* workspace, size_t workspace_bytes,
                       const void* W_UV, void* o_lat, float* lse, void* out,
                       int B, int H, int d_c, int d_head, int num_splits,
                       mla_dtype io_dtype, unsigned flags, void* hip_stream);

/*
 * mla_merge_out_proj after mla_decode_paged_multi(..., MLA_FLAG_SKIP_MERGE)
 * with the same B, q_len, heads, d_c, num_splits and workspace:
 *   o_lat [B, q_len, heads, d_c], lse [B, q_len, heads] (may be NULL),
 *   out   [B, q_len, heads, d_head];  W_UV [heads, d_c, d_head].
 * mla_merge_out_proj is this call with q_len 1.
 */
int mla_merge_out_proj_multi(const void* workspace, size_t workspace_bytes,
                             const void* W_UV, void* o_lat, float* lse, void* out,
                             int B, int q_len, int heads, int d_c, int d_head,
                             int num_splits, mla_dtype io_dtype, unsigned flags,
                             void* hip_stream);

/*
 * Bytes of device workspace mla_prefill_mha needs: the concatenated per-head
 * projections, the materialised keys and values (B * heads * max_pages_per_seq
 * pages of 64 rows of 320 bf16 values: 40 KB per page and head), and the page
 * table and lengths of the (sequence, head) pairs.  Pure host function; 0 if an
 * argument is invalid.
 */
size_t mla_prefill_workspace_bytes(int B, int heads, int d_c, int max_pages_per_seq);

/*
 * Prefill in the "MHA paradigm" (Sec. 3.3, first of the two side-by-side
 * attention equations; the text before them names it the form for the
 * compute-intensive phase): keys and values are materialised per head from the
 * cached latent rows,
 *     k_{j,h} = [ W^{UK}_h c_j ; k^R_j ],     v_{j,h} = W^{UV}_h c_j,
 * and query token i of q_len (position seq_lens[b] - q_len + i; the cache
 * already holds the rows of all q_len tokens, as for mla_decode_paged_multi)
 * attends to the keys 0 .. its own position:
 *     out[b,i,h,:] = sum_j softmax_j( [q_nope ; q_rope] . k_{j,h} * scale ) v_{j,h}.
 * q_len = seq_len is the prefill of a whole prompt, q_len < seq_len a later
 * chunk of it.  Same function as mla_absorb_q -> mla_decode_paged_multi ->
 * mla_out_proj, at (2 (d_head + d_rope) + 2 d_head) instead of
 * (2 (d_c + d_rope) + 2 d_c) flop per (query, key, head), plus the
 * materialisation, 4 d_c d_head flop per (key, head).
 *
 *   q_nope [B, q_len, heads, d_head]   q_rope [B, q_len, heads, d_rope]   io dtype
 *   W_UK   [heads, d_head, d_c]        W_UV   [heads, d_c, d_head]
 *   kv_cache, page_table, seq_lens     as for mla_decode_paged
 *   out    [B, q_len, heads, d_head] io dtype (output); tokens that see no key
 *          (seq_len < q_len) give zeros
 *   lse    [B, q_len, heads] fp32 (output, may be NULL)
 *   workspace  mla_prefill_workspace_bytes(B, heads, d_c, max_pages_per_seq)
 *          bytes, 256-byte aligned; scratch
 * The materialised keys and values are rounded to bf16 (a rounding the absorbed
 * form does not have).  Supported: BF16 io and cache, d_head 128, d_rope 64,
 * page_size 64, d_c 256 or 512, B * heads <= 65535; otherwise
 * MLA_ERR_UNSUPPORTED (use the absorbed calls).
 */
int mla_prefill_mha(const void* q_nope, const void* q_rope,
                    const void* W_UK, const void* W_UV,
                    const void* kv_cache, const int32_t* page_table,
                    const int32_t* seq_lens, void* out, float* lse,
                    void* workspace, size_t workspace_bytes,
                    int B, int q_len, int heads, int d_head, int d_c, int d_rope,
                    int page_size, int num_pages, int max_pages_per_seq,
                    float softmax_scale, mla_dtype io_dtype,
                    mla_dtype cache_dtype, void* hip_stream);

/*
 * Bytes of device workspace mla_cache_append needs (fp32 partial rows of the
 * projection, one per slice of the model dimension).  Pure host function;
 * returns 0 if an argument is invalid.
 */
size_t mla_append_workspace_bytes(int B, int D, int d_c, int d_rope, mla_dtype io_dtype);

/*
 * Cache append: produces and stores the cache row of one new token per
 * sequence (Sec. 3.3, MLA equations: c^{KV}_t = W^{DKV} x_t,
 * k^R_t = RoPE(W^{KR} x_t, t); App. D.2: the latent is what the cache keeps;
 * RoPE as in Sec. 3.1 Eq. 1, consecutive (real, imaginary) pairs, pair i
 * turned by t * rope_base^(-2i/d_rope)):
 *
 *   row_b = [ x_b . W[:, :d_c]  |  RoPE( x_b . W[:, d_c:], positions[b] ) ]
 *
 * written to logical position positions[b] of sequence b, i.e. row
 * positions[b] % page_size of page page_table[b][positions[b] / page_size].
 * The caller passes positions[b] = the sequence's length before the append
 * and raises its seq_lens afterwards; the page must already be in the table.
 *
 *   x          [B, D] io dtype: the hidden state of the new token
 *   W_DKVR     [D, d_c + d_rope] io dtype: columns 0..d_c-1 are (W^{DKV})^T,
 *              the rest (W^{KR})^T
 *   kv_cache   pool as in mla_decode_paged (cache dtype); only the B rows
 *              named above are written
 *   kv_scale   [num_pages, page_size] fp32: required iff the cache dtype is
 *              MLA_FP8_E4M3: receives absmax(row)/448 (1 for an all-zero
 *              row); the codes are round-to-nearest-even of row/scale,
 *              saturating at +-448.  NULL otherwise.
 *   positions  [B] int32.  A position outside [0, max_pages_per_seq *
 *              page_size), or a page id outside [0, num_pages), is not an
 *              error code (both are device memory): that sequence is skipped.
 *   workspace  at least mla_append_workspace_bytes(...) bytes, 16-byte aligned
 *
 * Rounding: fp32 accumulation, one rounding to the cache dtype; the rotation
 * angle is formed in fp64.  d_rope even, d_c + d_rope <= 1024; any B, D.
 */
int mla_cache_append(const void* x, const void* W_DKVR, void* kv_cache, float* kv_scale,
                     const int32_t* page_table, const int32_t* positions,
                     void* workspace, size_t workspace_bytes,
                     int B, int D, int d_c, int d_rope, int page_size,
                     int num_pages, int max_pages_per_seq, float rope_base,
                     mla_dtype io_dtype, mla_dtype cache_dtype, void* hip_stream);

/*
 * Test hook: the logical (un-paged) view of the cache, byte for byte, using
 * the same page arithmetic as mla_decode_paged.
 *
 *   dense [B, max_len, row_bytes] bytes (output): row j of sequence b is the
 *         row_bytes bytes of its cache row for j < seq_lens[b], else zeros.
 * row_bytes must be a multiple of 4.  Page ids outside [0, num_pages) give
 * zero rows.
 */
int mla_gather_paged(const void* kv_cache, const int32_t* page_table,
                     const int32_t* seq_lens, void* dense,
                     int B, int max_len, int row_bytes, int page_size,
                     int num_pages, int max_pages_per_seq, void* hip_stream);

/*
 * Diagnostic: how fast one launch of the bf16 decode kernel's shape can stream
 * a cache at all.  Runs the tile requests, counted waits and per-tile barriers
 * of the kernel mla_decode_paged uses for short uniform chunks (grid B x
 * num_splits, ring of four 36 KB tiles per workgroup, non-temporal
 * direct-to-LDS loads) with no query rows, no arithmetic and no output: the
 * time of a launch is what Sec. 3.3's second line costs on this part when
 * everything but reading the cached rows once is free.  bench.py reports it
 * beside the decode kernel's time.
 *
 *   kv_cache   [num_pages, 64, d_c + 64] bf16 (device), d_c 256 or 512
 *   page_table [B, max_pages_per_seq] int32, seq_lens [B] int32 (device)
 *   num_splits chunks per sequence, as for mla_decode_paged
 *
 * Reads only; page ids outside [0, num_pages) are skipped.  Returns MLA_OK or
 * an error code as the other calls do; allocates nothing.
 */
int mla_diag_stream_tiles(const void* kv_cache, const int32_t* page_table, const int32_t* seq_lens,
                          int B, int d_c, int num_pages, int max_pages_per_seq, int num_splits,
                          void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MLA_GFX950_H */
