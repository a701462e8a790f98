// Matrix-core paged decode for an fp8 (OCP e4m3) latent cache with one fp32 scale per row
// (gfx950 / CDNA4): every contraction runs on the cached codes as they are.
//
// Second line of the absorbed attention equation (Sec. 3.3 of the paper): all H heads score
// against the ONE shared row k_hat_j = [c_j ; k^R_j] and weight the same latent rows c_j:
//     S^T [tok x heads]   = K [tok x (d_c+64)] . Q^T [(d_c+64) x heads]
//     O^T [d_c x heads]  += V^T [d_c x tok] . P^T [tok x heads]
// with V = the first d_c columns of the very same LDS tile as K.  A tile is a whole page of codes
// (64 rows x (d_c + 64) bytes) and travels raw, by direct-to-LDS loads, through a ring of four
// slots; the rows' scales follow by a 4-byte direct-to-LDS load per row.
//
// The instruction is v_mfma_scale_f32_16x16x128_f8f6f4 (128 e4m3 products per lane pair and
// instruction, twice the rate of the bf16 instructions, one power-of-two block scale per 32 k).
// What is not e4m3 by nature is written as TWO e4m3 terms, hi + lo, with a power-of-two unit:
//   query rows : q / s = hi + lo, s per head such that the head's largest element lands in
//                [128, 256): together 2^-8 relative, the precision of the bf16 element itself;
//   weights    : w 2^c = hi + lo for w = 2^(x - m) * (the row's scale), c per block of 32 weights
//                such that their largest lands in [128, 256); 2^-c goes back in as the
//                instruction's block scale, so weights of any magnitude keep 2^-8 relative to
//                the largest of their block.  The normaliser sums the plain weights 2^(x - m).
// No cached element is ever converted.
//
// Eight wavefronts, two per SIMD, of two kinds that meet at one workgroup barrier per tile:
//   wavefronts 4..7, S (hg, hh): request the tiles (nine 128-bit loads per tile each, awaited by
//     count) and turn tile t into weights: scores of the 32 rows of tile half hh against the 16
//     heads of head group hg (18 instructions), scaling, masks, reference, exponentials, the
//     two-term split; the weights go to LDS (16 bytes per lane, two buffers);
//   wavefronts 0..3, V (hg, ch): accumulate O^T for heads 16 hg .. + 15 and latent columns
//     [ch d_c/2, (ch+1) d_c/2): one tile behind, they contract tile t - 1 with its weights (one
//     instruction per column tile, fed by two 8-bit transposing reads) while S works on tile t.
// A single wavefront issues in order and has 256 registers; one that scored AND accumulated
// (as the bf16 kernel's consumers do) spent its time on LDS read issue and on moving data
// between the two jobs, and recomputed every score in both column halves.
//
// The two S wavefronts of a head group need the same reference m for a head.  Fast pass: the
// reference is the maximum of the head's first tile with a visible row; until every head has
// one, both score both halves (same data, same decisions), afterwards each its own.  A later
// score more than FAST_GAP above the reference raises a flag, and the chunk is done again by the
// careful pass (rare), where both always score both halves, the reference moves whenever a
// tile's maximum exceeds it by more than RESCALE_GAP, and the factor for the accumulators
// travels with the weights.
#include "mla_internal.h"
#include "mfma_tile.h"
#include <type_traits>

namespace mla {
namespace {

constexpr int SF_THREADS = 512;   // 4 V + 4 S wavefronts

typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(8))) int i32x8;

// s_waitcnt vmcnt(min(younger, N))
template <int N>
__device__ __forceinline__ void wait_at_most(int younger)
{
    if (younger >= N) wait_vmcnt<N>();
    else if constexpr (N > 0) wait_at_most<N - 1>(younger);
}

// BAL = true: the balanced partition (one-dimensional grid; a workgroup owns an equal share of the
// pages of all sequences laid end to end and runs its segments one after the other, see
// decode_mfma.hip, whose plan and slot numbering this is).
template <int D_C, bool BAL>
__global__ __launch_bounds__(SF_THREADS, 1) void decode_stream_fp8_kernel(DecodeParams p)
{
    constexpr int LOOK = 2;                     // tiles requested beyond the one being scored
    constexpr int RING = 4;                     // ring slots: LOOK + 1, and one more: tile t - 1 is still being contracted
    constexpr int ROWB = D_C + 64;              // bytes per cached row
    constexpr int CPR = ROWB / 16;              // 16-byte chunks per cached row (36 / 20)
    constexpr int PAGE_B = 64 * ROWB;           // bytes per page = per tile
    constexpr int TR = 64;                      // cached rows per tile
    constexpr int TILE_B = PAGE_B;
    constexpr int QROWB = ROWB * 2;             // bytes per query row (bf16)
    constexpr int QCPR = QROWB / 16;            // 16-byte chunks per query row
    static_assert(32 * QROWB == TILE_B, "the 32 query rows are loaded like one tile");
    constexpr int NLOAD = TILE_B / (256 * 16);  // 16-byte loads per S thread per tile (9 / 5)
    constexpr int NJ = D_C / 128;               // 128-element k-groups of the latent part (4 / 2)
    constexpr int WCT = D_C / 32;               // column tiles of the value contraction per V wavefront (16 / 8)
    constexpr int RSO = WCT * 32 + 32;          // epilogue: row stride of the transposed block in bytes (padded)
    constexpr int A_STEP = 128;                 // bytes from k-group j to j + 1
    constexpr int V_STEP = 64;                  // bytes from column tile ct to ct + 4
    constexpr int ONE = 0x7F7F7F7F;             // block scale 2^0 in every byte
    static_assert(TILE_B % (256 * 16) == 0, "tile must split evenly over the loads");
    static_assert(QCPR % 8 == 0 && CPR % 2 == 0, "the chunk swizzles need rows of whole groups of chunks");
    static_assert((NLOAD + 1) * (LOOK + 1) < 64, "vmcnt is a 6-bit counter");
    static_assert(4 * 16 * RSO <= 3 * TILE_B, "the epilogue's transposition space must fit in the tile ring");

    // four tile slots: slot 3 receives the query rows first and joins the ring afterwards (its first
    // tile is requested after the first barrier but one, when the query rows are in registers)
    __shared__ __attribute__((aligned(1024))) unsigned char smem[RING * TILE_B];
    __shared__ float sc_lds[RING][64];            // the row scales of the tiles in the ring
    __shared__ u32x4 w_lds[2][2][2][64];          // weights [tile parity][head group][tile half][lane]: first term (8 bytes), second term (8 bytes)
    __shared__ uint32_t ws_lds[2][2][2][2][16];   // their block scales [parity][head group][half][pair of lane groups][head], e8m0 in every byte
    __shared__ float fa_lds[2][2][16];            // careful pass: factor for the accumulators [parity][head group][head]
    __shared__ float l_lds[2][2][16];             // the normaliser's parts [head group][half][head]
    __shared__ float m_lds[2][16];                // the references [head group][head]
    __shared__ int jump_flag;                     // raised by an S wavefront whose fast pass met a score far above its reference
    __shared__ int seg_lds[BAL ? 64 : 1][3];      // balanced partition: this workgroup's segments within a block of 64 sequences
    LDS_AS unsigned char* lds = (LDS_AS unsigned char*)smem;

    const int tid = (int)threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroup -> query-row group and (sequence, chunk): as in decode_mfma.hip (groups of 32 query
    // rows beyond the first go to further workgroups, 8 linear ids apart: same XCD, shared L2).
    const int Z = (p.H + 31) / 32;
    int wg_lin = blockIdx.x, zi = 0;
    if (Z > 1) {
        const int id = blockIdx.x, r = id >> 3;
        zi = r % Z;
        wg_lin = (r / Z) * 8 + (id & 7);
        if (wg_lin >= p.B * p.num_splits) return;   // padding of the last group of 8
    }
    const int hb = zi * 32;
    const bool stream_once = Z == 1;   // no other workgroup reads this one's cached rows

    // one chunk (uniform partition) or one segment (balanced: rows [seg_row0, seg_row1) of sequence b,
    // partials into slot out_slot)
    auto run_segment = [&](const int b, const int split, const int seg_row0, const int seg_row1,
                           const size_t out_slot) {
    // (balanced partition: everything derived from the thread index is derived again per segment
    // from a value the compiler cannot see through, so that it is not kept in registers across
    // segments)
    int opaque_zero = 0;
    if constexpr (BAL) asm volatile("" : "+v"(opaque_zero));
    const int tid = (int)threadIdx.x + opaque_zero;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool swave = wave >= 4;              // S: loads, scores, weights;  V: value contraction
    const int w4 = wave & 3;
    const int hg = w4 & 1;                     // head group (both kinds)
    const int ch = w4 >> 1;                    // V: column half
    const int hh = w4 >> 1;                    // S: tile half
    const int n = lane & 15, g = lane >> 4;
    const int head = hg * 16 + n;
    const int HL = min(32, p.H - hb);          // query rows of this workgroup
    if (tid == 0) jump_flag = 0;               // read after the tile loop, behind at least one barrier
    auto o_row = [&](int h) -> uint16_t* {     // partial rows are bf16 (the io dtype of this kernel)
        return static_cast<uint16_t*>(p.o_part) + (BAL ? (out_slot * p.H + h) : part_index(b, h, split, p.H, p.num_splits)) * D_C;
    };
    auto lse_at = [&](int h) -> float* {
        return p.lse_part + (BAL ? (out_slot * p.H + h) : part_index(b, h, split, p.H, p.num_splits));
    };

    // read-only tables go through the scalar cache
    const CONST_AS int32_t* seq_lens_c = (const CONST_AS int32_t*)p.seq_lens;
    const CONST_AS int32_t* ptab = (const CONST_AS int32_t*)(p.page_table + (size_t)b * p.max_pages);
    const int warm = ptab[min(BAL ? seg_row0 / 64 : split * p.chunk_pages, p.max_pages - 1)];
    int L = seq_lens_c[b];
    asm volatile("" :: "s"(warm));
    L = max(0, min(L, p.max_pages * 64));
    const int row0 = BAL ? seg_row0 : split * p.chunk_pages * 64;                  // first cached row of this chunk
    const int row1 = BAL ? min(seg_row1, L) : min(row0 + p.chunk_pages * 64, L);   // one past its last row
    if (row0 >= row1) {  // empty chunk: weight zero in the merge, partial output never read
        if (tid < HL) *lse_at(hb + tid) = -INFINITY;
        return;
    }
    const int t0 = row0 / TR;                                     // tiles [t0, t1) of the sequence
    const int t1 = (row1 + TR - 1) / TR;

    // Chunk swizzle of a cached row in LDS (applied on the global-address side of the loads: LDS chunk
    // position pc of row r holds the row's chunk pc ^ key(r)).  Rows are 64 bytes mod 256 long, so
    // rows 4 apart share a quarter of the 256-byte bank window.  A 128-bit LDS read is served 16
    // lanes at a time (lanes 0-7 with 24-31, 8-15 with 16-23, and the same in the upper half:
    // measured), the score reads touch rows {8i + 4bk + j} with two adjacent lane groups two chunks
    // apart, the transposing reads rows 8g .. 8g+7 at one chunk index; this 1-bit key (it stays inside
    // aligned pairs of chunks) puts the rows that meet in one such service on different positions:
    // the score reads run at the rate LDS delivers bytes (measured: 31.8 cycles per instruction with
    // four wavefronts reading, against 32 for conflict-free reads), the transposing reads within a
    // quarter of it (19.8 against 16).
    auto row_key = [](int r) { return (r >> 3) & 1; };
    // rows of tile t that belong to this chunk (0 if its page id is outside the pool)
    auto rows_valid = [&](int t) {
        const int page = ptab[t];
        return (page >= 0 && page < p.num_pages) ? min(TR, row1 - t * TR) : 0;
    };
    // first cached row (of the sequence) that some query row of the sequence must not see
    const int causal_from = L - (p.q_len - 1);

    // ================================================================== loads (both kinds)
    // HBM -> LDS with direct-to-LDS 128-bit loads (inline assembly: the compiler keeps no record of
    // them).  Load k of the wavefronts with index w (= wave % 4) fills LDS chunks [(4k+w)*64, +64) of
    // the tile; LDS chunk P = row r, position pc holds the row's chunk pc ^ key(r).  A load leaves the
    // wavefront that issues it standing in the memory pipe's queue until the request is accepted,
    // with the memory system saturated about 200 cycles: the loads of a tile are therefore shared
    // out so that both kinds of wavefront are busy for about as long per tile (measured: V contracts
    // for 1470 cycles, S scores and weighs for 1910): V issues loads k < NLV, S the rest and the
    // scales.  The byte offset of a thread's k-th chunk is worked out anew for every tile from a lane
    // index the compiler cannot see through (kept in registers it would be live across everything
    // else these wavefronts do).
    constexpr int NLV = (NLOAD * 5 + 4) / 9;     // 5 of 9 / 3 of 5
    const int k_first = swave ? NLV : 0, k_last = swave ? NLOAD : NLV;   // this wave's loads of a tile
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    auto chunk_offset = [&](int k, int lane_o) -> uint32_t {
        const int P = (k * 4 + w4) * 64 + lane_o;
        const int r = P / CPR, pc = P % CPR;
        return (uint32_t)(r * ROWB + ((pc ^ row_key(r)) << 4));
    };
    const unsigned char* kv = static_cast<const unsigned char*>(p.kv);
    // returns the number of loads this thread issued (uniform)
    auto fetch_tile = [&](int t) -> int {
        if (rows_valid(t) <= 0) return 0;   // a page outside the pool is never dereferenced
        const int page = ptab[t];
        const unsigned char* src = kv + (size_t)page * PAGE_B;
        const uint32_t dst = lds_base + (uint32_t)(((t - t0) % RING) * TILE_B + w4 * 1024);
        int lane_o = lane;
        asm volatile("" : "+v"(lane_o));
        if (swave && w4 == 0) {   // the page's 64 row scales: one 4-byte direct-to-LDS load per lane
            const float* sp = p.kv_scale + ((size_t)page * 64 + lane_o);
            const uint32_t m0s = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(LDS_AS float*)&sc_lds[(t - t0) % RING][0]);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
                         :: "s"(m0s), "v"(sp) : "memory");
        }
        if (stream_once) {
            // this workgroup is the only reader of these rows: non-temporal loads
#pragma unroll
            for (int k = 0; k < NLOAD; ++k) {
                if (k < k_first || k >= k_last) continue;
                const unsigned char* gp = src + chunk_offset(k, lane_o);
                const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst + k * 4096);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
                             :: "s"(m0v), "v"(gp) : "memory");
            }
        } else {
            // further groups of query rows read the same rows from this XCD's L2: ordinary loads
#pragma unroll
            for (int k = 0; k < NLOAD; ++k) {
                if (k < k_first || k >= k_last) continue;
                const unsigned char* gp = src + chunk_offset(k, lane_o);
                const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst + k * 4096);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                             :: "s"(m0v), "v"(gp) : "memory");
            }
        }
        return (k_last - k_first) + ((swave && w4 == 0) ? 1 : 0);
    };
    // wait until at most `younger` of this wave's loads are outstanding (the count is an immediate of
    // the instruction, hence the chain of cases)
    auto wait_younger = [&](int younger) { wait_at_most<2 * NLOAD + 2>(younger); };
    // the query rows [q_abs | q_rope] of the 32 heads into slot 3, laid out like 32 rows of a bf16
    // tile (one row per head, mfma_tile.h's chunk swizzle; rows of absent heads zero-filled)
    LDS_AS unsigned char* qlds = lds + 3 * TILE_B;
    auto fetch_query_rows = [&]() {
        const unsigned char* qa = static_cast<const unsigned char*>(p.q_abs) + ((size_t)b * p.H + hb) * D_C * 2;
        const unsigned char* qr = static_cast<const unsigned char*>(p.q_rope) + ((size_t)b * p.H + hb) * 128;
        const uint32_t dst = (uint32_t)(uintptr_t)qlds + (uint32_t)(w4 * 1024);
#pragma unroll
        for (int k = 0; k < NLOAD; ++k) {
            const int P = (k * 4 + w4) * 64 + lane;
            const int r = P / QCPR, c = (P % QCPR) ^ swz_key(r);
            if (r < HL) {
                const unsigned char* gp = c < D_C / 8 ? qa + ((size_t)r * D_C + c * 8) * 2
                                                      : qr + ((size_t)r * 64 + (c - D_C / 8) * 8) * 2;
                const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst + k * 4096);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                             :: "s"(m0v), "v"(gp) : "memory");
            } else {
                *(LDS_AS u32x4*)(qlds + P * 16) = (u32x4){0u, 0u, 0u, 0u};
            }
        }
    };
    // the first requests of a pass: (the query rows,) the first tile and the one after it.  Returns
    // the number of loads this wave issued for the first tile; first_ahead = for the second.
    int first_ahead = 0;
    auto request_first = [&](bool with_query_rows) -> int {
        if (with_query_rows && swave) fetch_query_rows();   // the oldest loads: every later wait covers them
        const int n0 = fetch_tile(t0);
        first_ahead = t0 + 1 < t1 ? fetch_tile(t0 + 1) : 0;
        return n0;
    };

    // ================================================================== S: scores and weights
    // Query operands (B), resident for the whole chunk.  Latent part: lane (g, n) holds elements
    // 128 j + 32 g .. + 31 of k-group j of head 16 hg + n, both terms.  Rope part (64 elements, half an
    // instruction's k): lane groups 0 and 1 hold the first term of elements 32 (g % 2) .. + 31, lane
    // groups 2 and 3 the second term of the same elements, so that one instruction contracts both.
    // A wavefront is S or V for life, and one register allocation serves both: the query operands
    // (72 / 40 registers) and V's accumulators (64 / 32) are therefore the SAME registers, st[], read
    // as 18 / 10 blocks of four: S takes operand i from st[2i], st[2i+1] (first terms: i = j, second
    // terms: i = NJ + j, rope: i = 2 NJ), V keeps the accumulator of column tile i in st[i].
    constexpr int NST = 4 * NJ + 2 > WCT ? 4 * NJ + 2 : WCT;
    f32x4 st[NST];
#pragma unroll
    for (int i = 0; i < NST; ++i) st[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    auto q_op = [&](int i) -> i32x8 {
        return __builtin_bit_cast(i32x8, __builtin_shufflevector(st[2 * i], st[2 * i + 1], 0, 1, 2, 3, 4, 5, 6, 7));
    };
    float q_unit = 1.f;        // s of this lane's head
    float m_run = -INFINITY;   // reference of the exponentials, scaled scores in log2 units
    float l_run = 0.f;         // this lane's share of the running sum (its 8 rows of every tile half it weighs)
    const float sc = p.scale * LOG2E;
    // maximum over the four lane groups, on every lane
    auto over_groups = [&](float v) {
        v = fmaxf(v, __shfl_xor(v, 16));
        return fmaxf(v, __shfl_xor(v, 32));
    };
    // Score A operand of block bk (16 of the half's 32 rows), lane (g, n): row 8 (n / 4) + n % 4 + 4 bk
    // of the half (so that D row 4g + i of block bk is half row 8g + 4bk + i: a lane's eight scores
    // are those of rows 8g .. 8g+7, the rows an 8-bit transposing read hands to lane group g), latent
    // part: bytes 128 j + 32 g .. + 31 (chunks 8j + 2g and 8j + 2g + 1) for k-group j; rope part: bytes
    // d_c + 32 (g % 2) .. + 31 (lane groups 2 and 3 read what 0 and 1 read: the codes meet the second
    // term of the query rows there).  Block 1's rows lie 4 rows behind block 0's and share their key.
    uint32_t ab[2], arb[2];
    {
        const uint32_t row = (uint32_t)((8 * (n >> 2) + (n & 3)) * ROWB), key = (uint32_t)((n >> 2) & 1);
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            ab[e] = row + (uint32_t)((g >> 1) * 64) + ((((uint32_t)((2 * g + e) & 3)) ^ key) << 4);
            arb[e] = row + (uint32_t)D_C + ((((uint32_t)(2 * (g & 1) + e)) ^ key) << 4);
        }
    }

    // S^T = K . Q^T for one half (32 rows, at `half`) x this wave's 16 heads, as a stream of A operands
    // (32 bytes per lane: two 128-bit reads): (k-group 0: block 0, block 1), ..., (k-group NJ-1: block 0,
    // block 1), rope: block 0, block 1; a latent operand feeds two instructions (the query rows' two
    // terms), a rope operand one (both terms at once).  An LDS read of this width takes about 200
    // cycles to come back (measured): the reads run three operands ahead.
    auto score_half = [&](LDS_AS unsigned char* half, LDS_AS const float* scales, int h, f32x4 (&sacc)[2], f32x4 (&rs)[2]) {
        constexpr int NO = 2 * NJ + 2;                       // operands of the half
        constexpr int D = 3;                                 // operands requested ahead
        u32x4 op[NO][2];
        auto ord = [&](int m) {
#pragma unroll
            for (int e = 0; e < 2; ++e)
                op[m][e] = m < 2 * NJ ? *(LDS_AS u32x4*)(half + ab[e] + (m & 1) * 4 * ROWB + (m >> 1) * A_STEP)
                                      : *(LDS_AS u32x4*)(half + arb[e] + (m - 2 * NJ) * 4 * ROWB);
        };
        sacc[0] = sacc[1] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int m = 0; m < D && m < NO; ++m) ord(m);
        // the rows' scales (lane (g, n): rows 8g .. 8g+7 of the half), needed right behind the last instruction
#pragma unroll
        for (int bk = 0; bk < 2; ++bk) rs[bk] = *(LDS_AS const f32x4*)(scales + h * 32 + 8 * g + 4 * bk);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NO; ++m) {
            if (m + D < NO) ord(m + D);
            const i32x8 k = __builtin_bit_cast(i32x8, __builtin_shufflevector(op[m][0], op[m][1], 0, 1, 2, 3, 4, 5, 6, 7));
            if (m < 2 * NJ) {
                sacc[m & 1] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(k, q_op(m >> 1), sacc[m & 1], 0, 0, 0, ONE, 0, ONE);
                sacc[m & 1] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(k, q_op(NJ + (m >> 1)), sacc[m & 1], 0, 0, 0, ONE, 0, ONE);
            } else {
                sacc[m - 2 * NJ] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(k, q_op(2 * NJ), sacc[m - 2 * NJ], 0, 0, 0, ONE, 0, ONE);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // the sums of half h of tile t -> scores in log2 units (times the rows' scales rs and
    // the power of two taken out of the query rows), rows outside the chunk or beyond the query row's
    // own position at -inf
    auto finish_half = [&](const f32x4 (&sacc)[2], const f32x4 (&rs)[2], int t, int h, int n_valid, float (&x)[2][4]) {
        const float unit = sc * q_unit;
        const int r0 = h * 32 + 8 * g;   // tile row behind D row 4g of block 0; block 1: 4 rows further
#pragma unroll
        for (int bk = 0; bk < 2; ++bk)
#pragma unroll
            for (int i = 0; i < 4; ++i) x[bk][i] = sacc[bk][i] * (unit * rs[bk][i]);
        if (n_valid < TR || (t + 1) * TR > causal_from) {
            const int seen = min(n_valid, visible_rows(p, L, hb + head) - t * TR);
#pragma unroll
            for (int bk = 0; bk < 2; ++bk)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (r0 + 4 * bk + i >= seen) x[bk][i] = -INFINITY;
        }
    };
    // one head's step from the scores of 32 rows to its reference; `factor` collects what the careful
    // pass's moves of the reference mean for everything accumulated before
    auto reference_step = [&](auto careful_tag, const float (&x)[2][4], bool& jumped, float& factor) {
        const float lmax = fmaxf(fmaxf(fmaxf(x[0][0], x[0][1]), fmaxf(x[0][2], x[0][3])),
                                 fmaxf(fmaxf(x[1][0], x[1][1]), fmaxf(x[1][2], x[1][3])));
        if constexpr (!decltype(careful_tag)::value) {
            if (__any(m_run == -INFINITY)) {       // first tile with a visible row (as a rule: the first tile)
                const float tmax = over_groups(lmax);
                if (m_run == -INFINITY) m_run = tmax;
            }
            jumped |= lmax > m_run + FAST_GAP;
        } else {
            const float tmax = over_groups(lmax);
            if (m_run == -INFINITY) m_run = tmax;  // nothing accumulated yet: nothing to rescale
            if (__any(tmax > m_run + RESCALE_GAP)) {
                const float m_new = tmax > m_run + RESCALE_GAP ? tmax : m_run;
                const float alpha = fast_exp2(m_run - m_new);   // 1 for the lanes that keep their reference
                l_run *= alpha;
                factor *= alpha;
                m_run = m_new;
            }
        }
    };
    // the weights of this wave's half: two e4m3 terms of w 2^c, into LDS.  The instruction's k order
    // (measured) puts the first 16 bytes of lane groups 2b and 2b+1 into scale block b and their
    // second 16 bytes into block 2 + b, and takes block kb's scale from lane group kb.  A V lane's 32
    // k slots are [half 0: first term, second term | half 1: first term, second term] of its rows
    // 8g .. 8g+7, so a block holds the 32 weights (both terms) that a PAIR of lane groups of ONE S
    // wavefront computes: c is the pair's, and it is stored per (half, pair, head) for the V lanes
    // of lane group 2 half + pair to pick up.
    auto weigh_half = [&](const float (&x)[2][4], const f32x4 (&rs)[2], int par) {
        const float m_use = m_run == -INFINITY ? 0.f : m_run;   // only while every row so far is masked
        float w[2][4], wmax = 0.f, lsum = 0.f;
#pragma unroll
        for (int bk = 0; bk < 2; ++bk)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float ex = fast_exp2(x[bk][i] - m_use);
                lsum += ex;
                w[bk][i] = ex * rs[bk][i];
                wmax = fmaxf(wmax, w[bk][i]);
            }
        l_run += lsum;
        // largest weight of the pair of lane groups (rows of 16 lanes: 0 with 1, 2 with 3)
        const u32x2 sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(wmax), __float_as_uint(wmax), false, false);
        wmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        const int c = min(134 - (int)(__float_as_uint(wmax) >> 23), 127);
        const float f = __uint_as_float((uint32_t)(c + 127) << 23);   // 2^c (c >= -121)
        uint32_t hi[2], lo[2];
#pragma unroll
        for (int bk = 0; bk < 2; ++bk) {
            const float v0 = w[bk][0] * f, v1 = w[bk][1] * f, v2 = w[bk][2] * f, v3 = w[bk][3] * f;
            int a = __builtin_amdgcn_cvt_pk_fp8_f32(v0, v1, 0, false);
            a = __builtin_amdgcn_cvt_pk_fp8_f32(v2, v3, a, true);
            const f32x2 b01 = __builtin_amdgcn_cvt_pk_f32_fp8(a, false);
            const f32x2 b23 = __builtin_amdgcn_cvt_pk_f32_fp8(a, true);
            int r = __builtin_amdgcn_cvt_pk_fp8_f32(v0 - b01[0], v1 - b01[1], 0, false);
            r = __builtin_amdgcn_cvt_pk_fp8_f32(v2 - b23[0], v3 - b23[1], r, true);
            hi[bk] = (uint32_t)a;
            lo[bk] = (uint32_t)r;
        }
        w_lds[par][hg][hh][lane] = (u32x4){hi[0], hi[1], lo[0], lo[1]};
        if ((g & 1) == 0) ws_lds[par][hg][hh][g >> 1][n] = (uint32_t)(127 - c) * 0x01010101u;   // 2^-c as an e8m0 block scale
    };
    // tile t: its weights into buffer `par`
    auto s_tile = [&](auto careful_tag, LDS_AS unsigned char* tile, LDS_AS const float* scales, int t, int n_valid,
                      int par, bool& jumped) {
        constexpr bool CAREFUL = decltype(careful_tag)::value;
        f32x4 sacc[2], rs[2];
        float x[2][4], factor = 1.f;
        // both halves while the reference is open (same data and same decisions in both wavefronts of
        // the head group), this wave's half otherwise
        const bool both = CAREFUL || __any(m_run == -INFINITY);
        if (both) {
            float xo[2][4];
            f32x4 rso[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                score_half(tile + h * 32 * ROWB, scales, h, sacc, rs);
                finish_half(sacc, rs, t, h, n_valid, x);
                reference_step(careful_tag, x, jumped, factor);
                if (h == hh) {
#pragma unroll
                    for (int bk = 0; bk < 2; ++bk) {
                        rso[bk] = rs[bk];
#pragma unroll
                        for (int i = 0; i < 4; ++i) xo[bk][i] = x[bk][i];
                    }
                }
            }
            weigh_half(xo, rso, par);
        } else {
            score_half(tile + hh * 32 * ROWB, scales, hh, sacc, rs);
            finish_half(sacc, rs, t, hh, n_valid, x);
            reference_step(careful_tag, x, jumped, factor);
            weigh_half(x, rs, par);
        }
        if constexpr (CAREFUL) {
            if (hh == 0 && g == 0) fa_lds[par][hg][n] = factor;
        }
    };

    // ================================================================== V: value contraction
    // O^T += V^T . P^T for the tile at vtile with the weights in buffer `par`, one instruction per
    // column tile.  Lane (g, n) supplies 8 bytes of row 8g + n / 2 of either half (columns 16 ct +
    // 8 (n % 2) ..: chunk ct, half n % 2) and receives rows 8g .. 8g+7 of column 16 ct + n; the
    // operand holds each half's 8 rows twice (register copy), against the weights' two terms.
    uint32_t vb[4];
    {
        const uint32_t base = (uint32_t)((8 * g + (n >> 1)) * ROWB + (n & 1) * 8), key = (uint32_t)(g & 1);
#pragma unroll
        for (int e = 0; e < 4; ++e) vb[e] = base + ((((uint32_t)e) ^ key) << 4);
    }
    auto v_tile = [&](auto careful_tag, LDS_AS unsigned char* vtile, int par) {
        constexpr int VP = 4;                   // column tiles whose reads are in flight
        u32x2 vv[WCT][2];
        auto value_read = [&](int i) {
            const int ct = ch * WCT + i;
            LDS_AS unsigned char* a = vtile + vb[ct & 3] + (ct >> 2) * V_STEP;
            vv[i][0] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2*)a));
            vv[i][1] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2*)(a + 32 * ROWB)));
        };
        const u32x4 p0 = w_lds[par][hg][0][lane], p1 = w_lds[par][hg][1][lane];
        // k slots [half 0: first term, second term | half 1: first term, second term]
        const i32x8 P = __builtin_bit_cast(i32x8, __builtin_shufflevector(p0, p1, 0, 1, 2, 3, 4, 5, 6, 7));
        const int sb = (int)ws_lds[par][hg][g >> 1][g & 1][n];   // block g = (half g / 2, pair g % 2)
#pragma unroll
        for (int i = 0; i < VP; ++i) value_read(i);
        if constexpr (decltype(careful_tag)::value) {
            const float alpha = fa_lds[par][hg][n];
#pragma unroll
            for (int i = 0; i < WCT; ++i) st[i] *= alpha;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < WCT; ++i) {
            if (i + VP < WCT) value_read(i + VP);
            const i32x8 a = __builtin_bit_cast(i32x8, __builtin_shufflevector(vv[i][0], vv[i][1], 0, 1, 0, 1, 2, 3, 2, 3));
            st[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, P, st[i], 0, 0, 0, ONE, 0, sb);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ================================================================== one pass over the chunk's tiles
    // In the interval behind the barrier of tile t: S turns tile t into weights (buffer t % 2) and
    // requests tile t + 2 (into the slot tile t - 2 has left); V contracts tile t - 1 with the weights
    // of buffer (t - 1) % 2.  Before the first tile V contracts it with weights zero (one contraction
    // that adds nothing, in exchange for a loop body without a case distinction).
    auto sweep = [&](auto careful_tag) -> bool {
        constexpr bool CAREFUL = decltype(careful_tag)::value;
        static_assert(LOOK == 2, "the first requests cover the first tile and the one after it");
        int ahead[LOOK];       // S: loads issued for the tiles after the one being awaited, oldest first
        ahead[0] = first_ahead;
        ahead[1] = 0;
        bool jumped = false;
        // weights zero in buffer 1 (nobody reads or writes it before the first barrier of the pass)
        if (swave) {
            w_lds[1][hg][hh][lane] = (u32x4){0u, 0u, 0u, 0u};
            if ((g & 1) == 0) ws_lds[1][hg][hh][g >> 1][n] = (uint32_t)ONE;
            if (CAREFUL && hh == 0 && g == 0) fa_lds[1][hg][n] = 1.f;
        }
        for (int t = t0; t < t1; ++t) {
            LDS_AS unsigned char* tile = lds + ((t - t0) % RING) * TILE_B;
            const int n_valid = rows_valid(t);
            // wait until my loads of tile t have landed (younger tiles may stay in flight)
            wait_younger(ahead[0] + ahead[1]);
            // tile t has landed (every wave's part), its predecessor's weights are in LDS, and V is done
            // with tile t - 2
            __syncthreads();
            {
                const int tn = t + LOOK;
                ahead[1] = tn < t1 ? fetch_tile(tn) : 0;
                ahead[0] = ahead[1];   // tile t + 1's loads are awaited next: only tile t + 2's are younger
                ahead[1] = 0;
            }
            if (n_valid < TR) {
                // ragged last tile (or a page id outside the pool): rows that are not part of the
                // sequence become zeros, and so do their scales, so that whatever they hold stays out
                for (int i = tid; i < (TR - n_valid) * CPR; i += SF_THREADS)
                    *(LDS_AS u32x4*)(tile + n_valid * ROWB + i * 16) = (u32x4){0u, 0u, 0u, 0u};
                if (tid >= n_valid && tid < TR) sc_lds[(t - t0) % RING][tid] = 0.f;
                __syncthreads();
            }
            if (swave) {
                s_tile(careful_tag, tile, (LDS_AS const float*)&sc_lds[(t - t0) % RING][0], t, n_valid, (t - t0) & 1, jumped);
            } else {
                // tile t - 1 (for the first tile: the tile itself, weights zero)
                v_tile(careful_tag, t > t0 ? lds + ((t - 1 - t0) % RING) * TILE_B : tile, (t - t0 + 1) & 1);
            }
        }
        __syncthreads();   // the last tile's weights are in LDS
        if (!swave) v_tile(careful_tag, lds + ((t1 - 1 - t0) % RING) * TILE_B, (t1 - 1 - t0) & 1);
        return jumped;
    };

    // ---- the query rows: requested first, awaited on their own (the tiles behind them stay in
    // flight), read by the S wavefronts behind a barrier of their own
    {
        const int n0 = request_first(true);
        if (swave) wait_younger(n0 + first_ahead);   // (V has no part in the query rows)
        __syncthreads();
    }
    if (swave) {
        const uint32_t q_row = (uint32_t)((hg * 16 + n) * QROWB);
        const uint32_t q_key = (uint32_t)swz_key(n);
        auto q_chunk = [&](int c) -> u32x4 {   // elements 8c .. 8c+7 of this lane's query row
            return *(LDS_AS u32x4*)(qlds + q_row + ((((uint32_t)c) ^ q_key) << 4));
        };
        // the head's largest magnitude -> the power of two s
        float amax = 0.f;
        auto chunk_max = [&](const u32x4 w) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                amax = fmaxf(amax, fmaxf(fabsf(__uint_as_float(w[k] << 16)), fabsf(__uint_as_float(w[k] & 0xFFFF0000u))));
        };
#pragma unroll
        for (int c = 0; c < 4 * NJ; ++c) chunk_max(q_chunk(16 * (c >> 2) + 4 * g + (c & 3)));
#pragma unroll
        for (int c = 0; c < 4; ++c) chunk_max(q_chunk(D_C / 8 + 4 * (g & 1) + c));
        amax = over_groups(amax);
        const int ef = min(max((int)(__float_as_uint(amax) >> 23) - 7, 1), 253);   // biased exponent of s
        q_unit = __uint_as_float((uint32_t)ef << 23);
        const float inv = __uint_as_float((uint32_t)(254 - ef) << 23);            // 1 / s
        // eight bf16 elements -> two registers of codes per term
        auto split8 = [&](const u32x4 w, int (&hi)[2], int (&lo)[2]) {
            float f[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                f[2 * k] = __uint_as_float(w[k] << 16) * inv;
                f[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u) * inv;
            }
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                hi[k] = __builtin_amdgcn_cvt_pk_fp8_f32(f[4 * k], f[4 * k + 1], 0, false);
                hi[k] = __builtin_amdgcn_cvt_pk_fp8_f32(f[4 * k + 2], f[4 * k + 3], hi[k], true);
                const f32x2 b01 = __builtin_amdgcn_cvt_pk_f32_fp8(hi[k], false);
                const f32x2 b23 = __builtin_amdgcn_cvt_pk_f32_fp8(hi[k], true);
                lo[k] = __builtin_amdgcn_cvt_pk_fp8_f32(f[4 * k] - b01[0], f[4 * k + 1] - b01[1], 0, false);
                lo[k] = __builtin_amdgcn_cvt_pk_fp8_f32(f[4 * k + 2] - b23[0], f[4 * k + 3] - b23[1], lo[k], true);
            }
        };
        // operand i, register r of its eight = st[2i + r / 4][r % 4]
        auto q_put = [&](int i, int r, int v) { st[2 * i + (r >> 2)][r & 3] = __builtin_bit_cast(float, v); };
#pragma unroll
        for (int c = 0; c < 4 * NJ; ++c) {
            int hi[2], lo[2];
            split8(q_chunk(16 * (c >> 2) + 4 * g + (c & 3)), hi, lo);
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                q_put(c >> 2, 2 * (c & 3) + k, hi[k]);
                q_put(NJ + (c >> 2), 2 * (c & 3) + k, lo[k]);
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            int hi[2], lo[2];
            split8(q_chunk(D_C / 8 + 4 * (g & 1) + c), hi, lo);
#pragma unroll
            for (int k = 0; k < 2; ++k) q_put(2 * NJ, 2 * c + k, g < 2 ? hi[k] : lo[k]);
        }
    }

    const bool jumped = sweep(std::false_type{});
    if (jumped) jump_flag = 1;
    __syncthreads();   // everybody is done with the last tile; nothing is in flight (the S wavefronts waited for it)
    if (__builtin_expect(jump_flag != 0, 0)) {
        // ---- careful pass (rare): the same chunk again with a moving reference
        m_run = -INFINITY;
        l_run = 0.f;
#pragma unroll
        for (int i = 0; i < WCT; ++i)
            if (!swave) st[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
        request_first(false);
        sweep(std::true_type{});
        __syncthreads();
    }

    // ---- the normaliser and the reference, from S to V
    if (swave) {
        float lt = l_run + __shfl_xor(l_run, 16);
        lt += __shfl_xor(lt, 32);
        if (g == 0) {
            l_lds[hg][hh][n] = lt;
            if (hh == 0) m_lds[hg][n] = m_run;
        }
    }
    __syncthreads();

    // ---- V: normalise and write the partial (bf16).  A V wavefront holds its column half of its 16
    // heads complete; a lane holds 4 consecutive columns of head n per column tile, which written
    // straight out would give 8-byte pieces, so the block is transposed through LDS (the tile ring
    // is free: every wave has passed a barrier after its last tile) and stored in whole runs of
    // half a latent row.
    if (!swave) {
        const float lt = l_lds[hg][0][n] + l_lds[hg][1][n];
        const float inv = lt > 0.f ? 1.f / lt : 0.f;
        LDS_AS unsigned char* mine = lds + w4 * (16 * RSO);
#pragma unroll
        for (int i = 0; i < WCT; ++i) {
            const f32x4 o = st[i] * inv;
            *(LDS_AS u32x2*)(mine + n * RSO + (i * 16 + g * 4) * 2) =
                (u32x2){pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
        }
        const int nrow = min(16, HL - hg * 16);
        constexpr int LPR = WCT * 2;             // lanes (of 16 bytes = 8 bf16) covering one row of the half (32 / 16)
        constexpr int RPI = 64 / LPR;            // rows one store instruction covers (2 / 4)
        // all reads first, then all stores, from one base address and a row stride
        const size_t row_stride = (size_t)(BAL ? 1 : p.num_splits) * D_C;   // elements between the partial rows of consecutive heads
        const int rl = lane / LPR, c = lane % LPR;
        uint16_t* dst0 = o_row(hb + hg * 16) + (size_t)rl * row_stride + ch * (WCT * 16) + c * 8;
        u32x4 v[16 / RPI];
#pragma unroll
        for (int j = 0; j < 16 / RPI; ++j) v[j] = *(LDS_AS u32x4*)(mine + (j * RPI + rl) * RSO + c * 16);
#pragma unroll
        for (int j = 0; j < 16 / RPI; ++j)
            if (j * RPI + rl < nrow)
                __builtin_nontemporal_store(v[j], reinterpret_cast<u32x4*>(dst0 + (size_t)(j * RPI) * row_stride));
        if (ch == 0 && head < HL && g == 0)
            *lse_at(hb + head) = lt > 0.f ? (m_lds[hg][n] + __builtin_amdgcn_logf(lt)) * LN2 : -INFINITY;
    }
    };  // run_segment

    if constexpr (!BAL) {
        // linear ids run over the sequences first, chunk by chunk, with the sequence rotated by the
        // chunk index (see decode_mfma.hip)
        const int cx = Z > 1 ? wg_lin % p.B : (int)blockIdx.x, cy = Z > 1 ? wg_lin / p.B : (int)blockIdx.y;
        run_segment((cx + cy) % p.B, cy, 0, 0, 0);
    } else {
        // ---- balanced partition, exactly as in decode_mfma.hip: pages of sequence b: P_b =
        // ceil(len_b / 64); workgroup w of G owns the global pages [P w / G, P (w+1) / G) of the
        // concatenation, P = sum_b P_b.  Every wavefront derives the same plan by itself (lanes stand
        // for sequences, 64 at a time, a wave scan gives each sequence's first and last global page);
        // workgroup 0 writes the plan for the merge, a workgroup with an empty range inside a
        // sequence's span marks its slot empty.
        const int wg = wg_lin, G = p.B * p.num_splits;
        auto seq_len_of = [&](int bb) { return bb < p.B ? max(0, min(p.seq_lens[bb], p.max_pages * 64)) : 0; };
        auto wave_scan = [&](int v) {                // inclusive prefix sum over the 64 lanes
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int u = __shfl_up(v, o);
                if (lane >= o) v += u;
            }
            return v;
        };
        int total = 0;
        for (int blk = 0; blk < p.B; blk += 64)
            total += __shfl(wave_scan((seq_len_of(blk + lane) + 63) >> 6), 63);
        total = __builtin_amdgcn_readfirstlane(total);
        const int ps = __builtin_amdgcn_readfirstlane((int)((long long)total * wg / G));
        const int pe = __builtin_amdgcn_readfirstlane((int)((long long)total * (wg + 1) / G));
        int carry = 0;
        for (int blk = 0; blk < p.B; blk += 64) {
            int nseg = 0;
            {
                const int bb = blk + lane;
                const int len = seq_len_of(bb);
                const int pg = (len + 63) >> 6;
                const int incl = carry + wave_scan(pg), excl = incl - pg;
                // workgroup of global page x: the largest w with P w / G <= x
                const int w0 = pg > 0 ? (int)((((long long)excl + 1) * G - 1) / total) : 0;
                const int w1 = pg > 0 ? (int)(((long long)incl * G - 1) / total) : -1;
                if (wg == 0 && wave == 0 && bb < p.B) {
                    // sequence bb's partials are the slots first .. first + cnt - 1 (slot of a segment
                    // = workgroup + sequence index: strictly increasing along the concatenation)
                    p.plan[2 * bb] = pg > 0 ? w0 + bb : 0;
                    p.plan[2 * bb + 1] = w1 - w0 + 1;
                }
                if (ps == pe && pg > 0 && wave == 0 && w0 <= wg && wg <= w1) {
                    for (int h = hb; h < min(p.H, hb + 32); ++h) p.lse_part[((size_t)wg + bb) * p.H + h] = -INFINITY;
                }
                const int lo = max(ps, excl), hi = min(pe, incl);
                const bool mine = pg > 0 && lo < hi;
                const unsigned long long mask = __ballot(mine);
                nseg = __builtin_popcountll(mask);
                if (mine && wave == 0) {
                    const int k = __builtin_popcountll(mask & ((1ull << lane) - 1ull));
                    seg_lds[k][0] = bb;
                    seg_lds[k][1] = (lo - excl) * 64;
                    seg_lds[k][2] = (hi - excl) * 64;     // clipped to the length inside the segment
                }
                carry = __builtin_amdgcn_readfirstlane(__shfl(incl, 63));
            }
            __syncthreads();
            for (int k = 0; k < nseg; ++k) {
                const int sb = seg_lds[k][0], r0 = seg_lds[k][1], r1 = seg_lds[k][2];
                run_segment(sb, 0, r0, r1, (size_t)wg + (size_t)sb);
                __syncthreads();   // the next segment reuses the LDS the epilogue just read
            }
            if (carry >= pe && wg != 0) break;   // nothing further overlaps (workgroup 0 goes on: it writes the plan)
            __syncthreads();                     // the list is rewritten for the next block
        }
    }
}

}  // namespace

hipError_t launch_decode_stream_fp8(const DecodeParams& p, dim3 grid, hipStream_t s, bool balanced)
{
    dim3 block(SF_THREADS);
    if (balanced && !p.plan) return hipErrorInvalidValue;
    if (p.d_c == 512 && balanced)      decode_stream_fp8_kernel<512, true><<<grid, block, 0, s>>>(p);
    else if (p.d_c == 512)             decode_stream_fp8_kernel<512, false><<<grid, block, 0, s>>>(p);
    else if (p.d_c == 256 && balanced) decode_stream_fp8_kernel<256, true><<<grid, block, 0, s>>>(p);
    else if (p.d_c == 256)             decode_stream_fp8_kernel<256, false><<<grid, block, 0, s>>>(p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace mla
