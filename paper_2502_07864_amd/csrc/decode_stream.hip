// Matrix-core paged decode for a bf16 latent cache, with the wavefronts that request cached rows
// kept apart from the wavefronts that consume them (gfx950 / CDNA4).
//
// Second line of the absorbed attention equation (Sec. 3.3 of the paper): all H heads score
// against the ONE shared row k_hat_j = [c_j ; k^R_j] and weight the same latent rows c_j:
//     S^T [tok x heads]   = K [tok x (d_c+64)] . Q^T [(d_c+64) x heads]
//     O^T [d_c x heads]  += V^T [d_c x tok] . P^T [tok x heads]
// with V = the first d_c columns of the very same LDS tile as K (see decode_mfma.hip for the
// operand layouts, the transposed formulation, the chunk swizzle and the fixed-reference fast
// pass with its careful second pass; this kernel shares all of them).
//
// What is different here is who does what.  A direct-to-LDS load leaves the wavefront that issues
// it standing in the memory pipe's queue until the request is accepted, and with the memory system
// saturated that is most of a tile period.  When the consuming wavefronts issue the requests
// themselves (decode_mfma.hip) they fall behind the rows that land meanwhile, and that backlog
// (ring depth - 1 tiles) is still to be consumed when the last request has gone out; their
// accumulators (all d_c columns for half the tile rows) also need a hand-over between the two row
// halves at the end, at one wavefront per SIMD.  Here a workgroup has eight wavefronts, two per
// SIMD:
//   wavefronts 4..7 (producers) do nothing but request tiles (nine 128-bit direct-to-LDS loads per
//     tile each) and wait for them by count;
//   wavefronts 0..3 (consumers) never touch the vector-memory counter.  Consumer (hg, ch) owns
//     heads 16 hg .. 16 hg + 15 and latent columns [ch d_c/2, (ch+1) d_c/2) for ALL 32 rows of a
//     tile: it scores both 16-row blocks (the score contraction is done twice per head group,
//     once per column half: the kernel has matrix-core time to spare, it is bound by the
//     memory stream) and accumulates its column half with K = 32 (one v_mfma_f32_16x16x32_bf16 per
//     column tile, fed by two transposing LDS reads).  Its 64 accumulator registers hold complete
//     sums, so the epilogue is normalise, transpose, store: no hand-over, no combine.
// Both kinds meet at one workgroup barrier per tile (tile t has landed, everybody is done with
// tile t - 1, whose slot the producers then fill again).
//
// FP8 = true: OCP e4m3 cache with one fp32 scale per row.  A tile is a whole page of codes (64 rows,
// the same 36 KB as 32 bf16 rows) and travels raw, by the same direct-to-LDS loads; the codes are
// widened exactly to bf16 where the consumers read their operands (8 codes per lane and MFMA:
// four v_cvt_scalef32_pk_bf16_fp8 with scale 1), so both contractions are the bf16 ones and LDS
// holds and delivers half the bytes.  The value operand comes from the 8-bit transposing read
// (ds_read_b64_tr_b8: lane 16g + n supplies 8 bytes of row 8g + n/2 and receives rows 8g .. 8g+7
// of column n: checked on the device), whose k order (k slot 8g + j = row 8g + j) the score
// contraction is made to match by which LDS row each of its operand lanes reads: block bk of a
// 32-row half scores rows 8i + 4bk .. 8i + 4bk + 3 (i = 0 .. 3), so that a lane's eight weights
// are those of rows 8g .. 8g+7.  A row's scale multiplies its score and rides on its weight.
#include "mla_internal.h"
#include "mfma_tile.h"
#include <type_traits>

namespace mla {
namespace {

constexpr int ST_THREADS = 512;   // 4 consumer + 4 producer wavefronts

typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(8))) int i32x8;

template <int D_C, bool FP8>
__global__ __launch_bounds__(ST_THREADS, 1) void decode_stream_kernel(DecodeParams p)
{
    constexpr int LOOK = 2;                     // tiles requested beyond the one being consumed
    constexpr int RING = FP8 ? 4 : 3;           // ring slots: LOOK + 1, and for fp8 one more: its consumers are still
                                                // reading tile t - 1 (value contraction) when they start on tile t
    constexpr bool BAL = false;                 // uniform chunks only; the balanced partition runs decode_mfma.hip's kernel
    constexpr int ROW = D_C + 64;               // elements per cache row
    constexpr int ROWB = ROW * (FP8 ? 1 : 2);   // bytes per cached row
    constexpr int CPR = ROWB / 16;              // 16-byte chunks per cached row (72 / 40; fp8: 36 / 20)
    constexpr int PAGE_B = 64 * ROWB;           // bytes per page
    constexpr int TR = FP8 ? 64 : 32;           // cached rows per tile (fp8: a whole page, bf16: half a page)
    constexpr int NH = TR / 32;                 // 32-row halves of a tile, consumed one after the other
    constexpr int TILE_B = TR * ROWB;           // bytes per tile (36864 / 20480 for either format)
    constexpr int QROWB = ROW * 2;              // bytes per query row (bf16)
    constexpr int QCPR = QROWB / 16;            // 16-byte chunks per query row
    static_assert(32 * QROWB == TILE_B, "the 32 query rows are loaded like one tile");
    constexpr int NLOAD = TILE_B / (256 * 16);  // 16-byte loads per producer thread per tile (9 / 5)
    constexpr int NKS = ROW / 32;               // k-steps of the score contraction (18 / 10)
    constexpr int NJ = D_C / 128;               // fp8: 128-element k-groups of the latent part (4 / 2)
    constexpr int WCT = D_C / 32;               // column tiles of the value contraction per consumer (16 / 8)
    constexpr int SG = NKS % 3 == 0 ? 3 : 2;    // k-steps per read-ahead group (score)
    constexpr int VG = 4;                       // column tiles per read-ahead group (value)
    constexpr int RSO = WCT * 32 + 32;          // epilogue: row stride of the transposed block in bytes (padded)
    static_assert(TILE_B % (256 * 16) == 0, "tile must split evenly over the producers' loads");
    static_assert(QCPR % 8 == 0 && CPR % (FP8 ? 4 : 8) == 0, "the chunk swizzles need rows of whole groups of chunks");
    static_assert((NLOAD + 1) * (LOOK + 1) < 64, "vmcnt is a 6-bit counter");
    static_assert(4 * 16 * RSO <= 3 * TILE_B, "the epilogue's transposition space must fit in the tile ring");

    // four tile slots: slot 3 receives the query rows first; for fp8 it then joins the ring (its
    // first tile is requested after the first barrier but one, when the query rows are in registers)
    __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * TILE_B];
    // the query rows [q_abs | q_rope] of the 32 heads, laid out exactly like a cache tile (one row per
    // head, same chunk swizzle): requested by the producers as direct-to-LDS loads right after the
    // first tile, read into registers by the consumers after the first barrier
    __shared__ float sc_lds[FP8 ? RING : 1][64];     // fp8: the row scales of the tiles in the ring
    // fp8: the rope part of the consumers' query operands (32 bytes per lane, as two arrays of 16-byte
    // pieces): read like a cached operand when its turn comes, it frees eight registers
    __shared__ u32x4 qr_lds[FP8 ? 4 : 1][2][64];
    __shared__ int jump_flag;                        // raised by a consumer whose fast pass met a score far above its reference
    LDS_AS unsigned char* lds = (LDS_AS unsigned char*)smem;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
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
    const bool producer = wave >= 4;
    const int w4 = wave & 3;
    const int hg = w4 & 1, ch = w4 >> 1;       // consumers: head group, column half
    const int n = lane & 15, g = lane >> 4;
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

    const int head = hg * 16 + n;
    // consumers: this wave's 16 query rows as B operands, resident for the whole chunk.
    //   bf16: lane (g, n) holds elements 8g .. 8g+7 of every 32-element k-step of head 16 hg + n.
    //   fp8 : as TWO e4m3 terms, q / s = hi + lo with s a power of two per head that brings the head's
    //         largest element into [128, 256) (hi = q / s rounded to e4m3, lo = the remainder rounded
    //         to e4m3: together 2^-8 relative, the precision of the bf16 element itself).  Latent
    //         part: lane (g, n) holds elements 128 j + 32 g .. + 31 of k-group j, both terms.  Rope
    //         part (64 elements, half an instruction's k): lane groups 0 and 1 hold the first term
    //         of elements 32 (g % 2) .. + 31, lane groups 2 and 3 the second term of the same
    //         elements, so that one instruction contracts both terms; this operand waits in LDS.
    bf16x8 qreg[FP8 ? 1 : NKS];
    i32x8 qhi[FP8 ? NJ : 1], qlo[FP8 ? NJ : 1];
    float q_unit = 1.f;   // fp8: s of this lane's head

    asm volatile("" :: "s"(warm));
    L = max(0, min(L, p.max_pages * 64));
    const int row0 = BAL ? seg_row0 : split * p.chunk_pages * 64;             // first cached row of this segment
    const int row1 = BAL ? min(seg_row1, L) : min(row0 + p.chunk_pages * 64, L);  // one past its last row
    if (row0 >= row1) {  // empty chunk: weight zero in the merge, partial output never read
        if (tid < HL) *lse_at(hb + tid) = -INFINITY;
        return;
    }
    const int t0 = row0 / TR;                                       // tiles [t0, t1) of the sequence
    const int t1 = (row1 + TR - 1) / TR;
    // Chunk swizzle of a cached row in LDS (applied on the global-address side of the loads: LDS
    // chunk position pc of row r holds the row's chunk pc ^ key(r)).  bf16: mfma_tile.h's key.
    // fp8: rows are 64 bytes mod 256 long, so rows 4 apart share a quarter of the 256-byte bank window.
    // A 128-bit LDS read is served 16 lanes at a time (lanes 0-7 with 24-31, 8-15 with 16-23, and the
    // same in the upper half: measured), the score reads touch rows {8i + 4bk + j} with two adjacent
    // lane groups two chunks apart, the transposing reads rows 8g .. 8g+7 at one chunk index; this
    // 1-bit key (it stays inside aligned pairs of chunks) puts the rows that meet in one such service
    // on different positions: the score reads run at the rate LDS delivers bytes (measured: 31.8
    // cycles per instruction with four wavefronts reading, against 32 for conflict-free reads), the
    // transposing reads within a quarter of it (19.8 against 16).  A second key bit from (r >> 2) & 1
    // would bring those to 19.1, at the price of an address register per row block.
    auto row_key = [](int r) { return FP8 ? ((r >> 3) & 1) : swz_key(r); };

    // rows of tile t that belong to this chunk (0 if its page id is outside the pool)
    auto rows_valid = [&](int t) {
        int page = ptab[FP8 ? t : t >> 1];
        return (page >= 0 && page < p.num_pages) ? min(TR, row1 - t * TR) : 0;
    };

    // ---- producers: tile staging, HBM -> LDS with direct-to-LDS 128-bit loads (inline assembly:
    // the compiler keeps no record of them).  Load k of producer w fills LDS chunks [(4k+w)*64, +64)
    // of the tile; LDS chunk P = row r, position pc holds the row's chunk pc ^ key(r).
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    // byte offset of this thread's k-th chunk inside a tile's rows.  Worked out anew for every tile
    // from a lane index the compiler cannot see through: kept in registers they would be live across
    // the consumers' code as well (one register allocation serves both roles), which has none to spare.
    auto chunk_offset = [&](int k, int lane_o) -> uint32_t {
        const int P = (k * 4 + w4) * 64 + lane_o;
        const int r = P / CPR, pc = P % CPR;
        return (uint32_t)(r * ROWB + ((pc ^ row_key(r)) << 4));
    };
    const unsigned char* kv = static_cast<const unsigned char*>(p.kv);
    // returns the number of loads this thread issued (0 or NLOAD; uniform)
    auto fetch_tile = [&](int t) -> int {
        if (rows_valid(t) <= 0) return 0;   // a page outside the pool is never dereferenced
        const int page = ptab[FP8 ? t : t >> 1];
        const unsigned char* src = kv + (size_t)page * PAGE_B + (FP8 ? (size_t)0 : (size_t)(t & 1) * TILE_B);
        const uint32_t dst = lds_base + (uint32_t)(((t - t0) % RING) * TILE_B + w4 * 1024);
        int lane_o = lane;
        asm volatile("" : "+v"(lane_o));
        if constexpr (FP8) {
            if (w4 == 0) {   // the page's 64 row scales: one 4-byte direct-to-LDS load per lane
                const float* sp = p.kv_scale + ((size_t)page * 64 + lane_o);
                const uint32_t m0s = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(LDS_AS float*)&sc_lds[(t - t0) % RING][0]);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
                             :: "s"(m0s), "v"(sp) : "memory");
            }
        }
        if (stream_once) {
            // this workgroup is the only reader of these rows: non-temporal loads
#pragma unroll
            for (int k = 0; k < NLOAD; ++k) {
                const unsigned char* gp = src + chunk_offset(k, lane_o);
                const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst + k * 4096);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
                             :: "s"(m0v), "v"(gp) : "memory");
            }
        } else {
            // further groups of query rows read the same rows from this XCD's L2: ordinary loads
#pragma unroll
            for (int k = 0; k < NLOAD; ++k) {
                const unsigned char* gp = src + chunk_offset(k, lane_o);
                const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst + k * 4096);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                             :: "s"(m0v), "v"(gp) : "memory");
            }
        }
        return NLOAD + ((FP8 && w4 == 0) ? 1 : 0);
    };
    // wait until at most `younger` of this wave's loads are outstanding (the largest count on the
    // list that does not exceed it; a tile is NLOAD loads, one more for the wave that fetches the scales)
    auto wait_younger = [&](int younger) {
        if (FP8 && younger >= 2 * NLOAD + 2) wait_vmcnt<2 * NLOAD + 2>();
        else if (younger >= 2 * NLOAD)       wait_vmcnt<2 * NLOAD>();
        else if (FP8 && younger >= NLOAD + 1) wait_vmcnt<NLOAD + 1>();
        else if (younger >= NLOAD)           wait_vmcnt<NLOAD>();
        else                                 wait_vmcnt<0>();
    };

    // producers: the query rows into their LDS area, chunk by chunk like a tile (rows of absent
    // heads zero-filled); requested once per segment, right after the first tile's loads
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

    // ---- consumers: running softmax state; this lane's head = column n of the D tiles; of every
    // 32-row half of a tile it owns 4 rows of each of the two 16-row score blocks (bf16: rows 4g + i
    // and 16 + 4g + i; fp8: rows 8g + i and 8g + 4 + i)
    float m_run = -INFINITY;   // reference of the exponentials, scaled scores in log2 units
    float l_run = 0.f;         // this lane's share of the running sum (its 8 rows per half)
    f32x4 oacc[WCT];
#pragma unroll
    for (int i = 0; i < WCT; ++i) oacc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const float sc = p.scale * LOG2E;
    // Score A operand of block bk, lane (g, n): one row of the half, elements 8 (4 ks + g) .. + 7.
    //   bf16: row 16 bk + n, 16-byte chunk 4 ks + g;
    //   fp8 : row 8 (n / 4) + n % 4 + 4 bk, 8 bytes: chunk 2 ks + g / 2, half g % 2.
    //         latent part: bytes 128 j + 32 g .. + 31 of the row (chunks 8j + 2g and 8j + 2g + 1) for
    //         k-group j; rope part: bytes d_c + 32 (g % 2) .. + 31 (lane groups 2 and 3 read what
    //         0 and 1 read: the codes meet the second term of the query rows there).
    // The swizzled chunk index splits into a per-lane part (low bits, xor-ed with the row's key; the
    // key is the same in both halves of a tile, and for bf16 in both blocks) and a compile-time part.
    uint32_t a_base[2][2];   // [block][bf16: k-step parity; fp8: first or second chunk of the lane's 32 bytes]
    uint32_t ar_base[2][2];  // fp8: [block][first or second chunk of the lane's 32 rope bytes]
#pragma unroll
    for (int bk = 0; bk < 2; ++bk) {
        const int a_r = FP8 ? 8 * (n >> 2) + (n & 3) + 4 * bk : 16 * bk + n;   // the lane's row of the half
        const uint32_t a_key = (uint32_t)row_key(a_r);
#pragma unroll
        for (int e = 0; e < 2; ++e)
            a_base[bk][e] = (uint32_t)(a_r * ROWB) +
                            (FP8 ? (uint32_t)((g >> 1) * 64) + ((((uint32_t)((2 * g + e) & 3)) ^ a_key) << 4)
                                 : ((((uint32_t)(4 * e + g)) ^ a_key) << 4));
#pragma unroll
        for (int e = 0; e < 2; ++e)
            ar_base[bk][e] = (uint32_t)(a_r * ROWB + D_C) + ((((uint32_t)(2 * (g & 1) + e)) ^ a_key) << 4);
    }
    if constexpr (FP8) {
        // block 1's rows lie 4 rows behind block 0's and share their key: said outright, so that one
        // register serves both (the difference goes into the reads' offset fields)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            a_base[1][e] = a_base[0][e] + 4 * ROWB;
            ar_base[1][e] = ar_base[0][e] + 4 * ROWB;
        }
    }
    constexpr int A_STEP = 128;                                    // bytes from k-step ks to ks + 2 (fp8: from k-group j to j + 1)
    // Value A operand (transposing reads), lane (g, n) supplies 8 bytes:
    //   bf16: row 4g + n / 4 of a 16-row block, element columns 16 ct + 4 (n % 4) ..: chunk 2 ct + (n % 4) / 2, half n % 2;
    //   fp8 : row 8g + n / 2 of the half, columns 16 ct + 8 (n % 2) ..: chunk ct, half n % 2 (the lane
    //         receives rows 8g .. 8g+7 of column 16 ct + n: its k slots, see the weights below).
    const int v_r = FP8 ? 8 * g + (n >> 1) : g * 4 + (n >> 2);
    const uint32_t v_key = (uint32_t)row_key(v_r);
    uint32_t v_base[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        v_base[e] = (uint32_t)(v_r * ROWB) + (uint32_t)((n & 1) * 8) +
                    (FP8 ? ((((uint32_t)e) ^ v_key) << 4)
                         : ((((uint32_t)(2 * e) + (uint32_t)((n & 3) >> 1)) ^ v_key) << 4));
    if constexpr (FP8) {   // (the same for the chunk positions 2 and 3 of the value reads)
        v_base[2] = v_base[0] + 32;
        v_base[3] = v_base[1] + 32;
    }
    constexpr int V_STEP = FP8 ? 64 : 128;                         // bytes from column tile ct to ct + 4
    // first cached row (of the sequence) that some query row of the sequence must not see
    const int causal_from = L - (p.q_len - 1);
    // maximum over the four lane groups, on every lane
    auto over_groups = [&](float v) {
        v = fmaxf(v, __shfl_xor(v, 16));
        return fmaxf(v, __shfl_xor(v, 32));
    };
    // S^T = K . Q^T for the two 16-row blocks x 16 heads of the half at `half`, bf16 cache: the MFMAs.
    // The two blocks' contractions are interleaved: each is a chain of MFMAs into one accumulator,
    // and a chain of this instruction on its own runs at its latency, not at its issue rate.
    auto score_bf16 = [&](LDS_AS unsigned char* half, f32x4& sacc0, f32x4& sacc1) {
        bf16x8 a0[NKS], a1[NKS];
        auto rd = [&](int ks) {
            a0[ks] = *(LDS_AS bf16x8*)(half + a_base[0][ks & 1] + (ks >> 1) * A_STEP);
            a1[ks] = *(LDS_AS bf16x8*)(half + a_base[1][ks & 1] + (ks >> 1) * A_STEP);
        };
#pragma unroll
        for (int ks = 0; ks < SG; ++ks) rd(ks);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s0 = 0; s0 < NKS; s0 += SG) {
#pragma unroll
            for (int ks = s0 + SG; ks < s0 + 2 * SG && ks < NKS; ++ks) rd(ks);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = s0; ks < s0 + SG && ks < NKS; ++ks) {
                sacc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[ks], qreg[ks], sacc0, 0, 0, 0);
                sacc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[ks], qreg[ks], sacc1, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // the contractions' sums -> scores in log2 units (fp8: times the rows' scales, returned in rs
    // and the power of two taken out of the query rows), rows outside the chunk or beyond the query
    // row's own position at -inf
    auto finish_scores = [&](const f32x4 sacc0, const f32x4 sacc1, LDS_AS const float* scales, int t, int h, int n_valid,
                             float (&x0)[4], float (&x1)[4], float (&rs0)[4], float (&rs1)[4]) {
        // tile row behind D row 4g of block 0 / block 1
        const int r0 = h * 32 + (FP8 ? 8 * g : 4 * g), r1 = r0 + (FP8 ? 4 : 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            rs0[i] = FP8 ? scales[r0 + i] : 1.f;
            rs1[i] = FP8 ? scales[r1 + i] : 1.f;
            x0[i] = sacc0[i] * (FP8 ? sc * q_unit * rs0[i] : sc);
            x1[i] = sacc1[i] * (FP8 ? sc * q_unit * rs1[i] : sc);
        }
        if (n_valid < TR || (t + 1) * TR > causal_from) {
            const int seen = min(n_valid, visible_rows(p, L, hb + head) - t * TR);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (r0 + i >= seen) x0[i] = -INFINITY;
                if (r1 + i >= seen) x1[i] = -INFINITY;
            }
        }
    };

    // bf16 cache: weights p = 2^(x - m_run) rounded to bf16: the lane's eight weights are the B
    // operand of the value contraction (K = 32: O^T += V^T . P^T over the half's 32 rows) as they
    // stand, k slot 8g + j being half row 4g + j (j < 4) or 16 + 4g + j - 4, which two 16-bit
    // transposing reads (one per 16-row block) deliver; the normaliser sums exactly the rounded weights.
    auto weights = [&](const float (&x0)[4], const float (&x1)[4]) -> bf16x8 {
        const float m_use = m_run == -INFINITY ? 0.f : m_run;  // only while every row so far is masked
        float e0[4], e1[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { e0[i] = fast_exp2(x0[i] - m_use); e1[i] = fast_exp2(x1[i] - m_use); }
        const uint32_t p01 = pack_bf16x2(e0[0], e0[1]), p23 = pack_bf16x2(e0[2], e0[3]);
        const uint32_t p45 = pack_bf16x2(e1[0], e1[1]), p67 = pack_bf16x2(e1[2], e1[3]);
        l_run += ((bf16_bits_to_f32(p01 & 0xFFFFu) + bf16_bits_to_f32(p01 >> 16)) +
                  (bf16_bits_to_f32(p23 & 0xFFFFu) + bf16_bits_to_f32(p23 >> 16))) +
                 ((bf16_bits_to_f32(p45 & 0xFFFFu) + bf16_bits_to_f32(p45 >> 16)) +
                  (bf16_bits_to_f32(p67 & 0xFFFFu) + bf16_bits_to_f32(p67 >> 16)));
        return __builtin_bit_cast(bf16x8, (u32x4){p01, p23, p45, p67});
    };

    // bf16 cache: O^T += V^T . P^T for the half at `half`
    auto value_bf16 = [&](LDS_AS unsigned char* half, const bf16x8 pb) {
        u32x2 lo[WCT], hi[WCT];
        auto rd = [&](int i) {
            const int ct = ch * WCT + i;
            LDS_AS unsigned char* a = half + v_base[ct & 3] + (ct >> 2) * V_STEP;
            lo[i] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)a));
            hi[i] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(a + 16 * ROWB)));
        };
#pragma unroll
        for (int i = 0; i < VG; ++i) rd(i);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c0 = 0; c0 < WCT; c0 += VG) {
#pragma unroll
            for (int i = c0 + VG; i < c0 + 2 * VG && i < WCT; ++i) rd(i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = c0; i < c0 + VG && i < WCT; ++i)
                oacc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    __builtin_bit_cast(bf16x8, (u32x4){lo[i][0], lo[i][1], hi[i][0], hi[i][1]}), pb, oacc[i], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // one head's step from the scores of 32 rows to its reference.  Fast pass: every head keeps the
    // maximum of its first tile with a visible row and only records whether a later score exceeded
    // it by more than FAST_GAP.  Careful pass: the reference moves (and the accumulators are
    // rescaled) whenever a maximum exceeds it by more than RESCALE_GAP.
    auto reference_step = [&](auto careful_tag, const float (&x0)[4], const float (&x1)[4], bool& jumped) {
        const float lmax = fmaxf(fmaxf(fmaxf(x0[0], x0[1]), fmaxf(x0[2], x0[3])),
                                 fmaxf(fmaxf(x1[0], x1[1]), fmaxf(x1[2], x1[3])));
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
#pragma unroll
                for (int i = 0; i < WCT; ++i) oacc[i] *= alpha;
                m_run = m_new;
            }
        }
    };

    // ---- fp8 cache.  Every contraction is a v_mfma_scale_f32_16x16x128_f8f6f4 on codes as they are
    // (no conversion of cached data anywhere; block scales 1 except the weights').  Per tile of 64
    // rows a consumer runs
    //   (1) the score contraction of the tile: S^T = K . Q^T as a stream of A operands (32 bytes per
    //       lane: two 128-bit reads), per half: (k-group 0: block 0, block 1), ..., (k-group NJ-1: block 0,
    //       block 1), rope: block 0, block 1; a latent operand feeds two instructions (the query rows' two
    //       terms), a rope operand one (both terms at once);
    //   (2) per half: sums -> scores in log2 units (times the rows' scales and the power of two taken
    //       out of the query rows), masks, the head's reference;
    //   (3) the value contraction of the tile BEFORE, O^T += V^T . P^T, one instruction per column tile:
    //       lane (g, n) owns rows 8g .. 8g+7 of both halves, its 32 k slots are [first term: half 0,
    //       half 1 | second term: half 0, half 1], and the value operand holds the same 16 rows (two
    //       8-bit transposing reads) twice (register copy);
    //   (4) the weights of this tile, which feed the next tile's (3): w = 2^(x - m_run) * (the row's
    //       scale) becomes two e4m3 terms of w 2^c; 2^-c goes back in as the instruction's block scale
    //       (an exact power of two, any exponent), so that weights of any magnitude keep 2^-8
    //       relative to the largest weight that shares their c.  The instruction's k order
    //       (measured) puts the first 16 bytes of lane groups 2b and 2b+1 into scale block b and
    //       their second 16 bytes into block 2 + b, and takes block kb's scale from lane group kb: c is
    //       therefore common to a pair of lane groups (32 weights, their largest in [128, 256)),
    //       and lane group kb supplies the scale of pair kb % 2.  The normaliser sums the plain weights.
    // (1) and (3) keep the matrix core busy, (2) and (4) the vector ALU, and a single wavefront
    // issues in order: in the fast pass the arithmetic of half 0 is therefore written into the
    // second half of (1) and that of half 1 into (3), slice by slice behind the matrix instructions
    // in whose shadow it runs.  The careful pass (rare) does the steps one after the other, (3)
    // first: its reference may move in (2), and the pending weights refer to the old one.
    // An LDS read of these widths takes about 200 cycles to come back (measured): the score
    // operands are requested three operands ahead, the value operands VP column tiles ahead, the
    // first of them during the end of (1).
    constexpr int VP = 4;
    constexpr int ONE = 0x7F7F7F7F;   // block scale 2^0 in every byte
    auto value_read = [&](LDS_AS unsigned char* vtile, const uint32_t (&vb)[4], int i, u32x2 (&r)[2]) {
        const int ct = ch * WCT + i;
        LDS_AS unsigned char* a = vtile + vb[ct & 3] + (ct >> 2) * V_STEP;
        r[0] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2*)a));
        r[1] = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_AS i32x2*)(a + 32 * ROWB)));
    };
    // one column tile of (3)
    auto value_step = [&](LDS_AS unsigned char* vtile, const uint32_t (&vb)[4], int i, u32x2 (&vv)[WCT][2], const i32x8 P, const int sb) {
        if (i + VP < WCT) value_read(vtile, vb, i + VP, vv[i + VP]);
        const i32x8 a = __builtin_bit_cast(i32x8, __builtin_shufflevector(vv[i][0], vv[i][1], 0, 1, 2, 3, 0, 1, 2, 3));
        oacc[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, P, oacc[i], 0, 0, 0, ONE, 0, sb);
        // (keeps the instruction, and the reads after it, where they are written: left to itself the
        // compiler moves contractions behind the softmax and their reads ahead of everything)
        asm volatile("" : "+v"(oacc[i]) :: "memory");
    };
    // the tile at `tile` (scores, weights) and the pending value contraction of the tile at vtile
    // (weights P, block scales sb, replaced by this tile's on return)
    auto fp8_tile = [&](auto careful_tag, LDS_AS unsigned char* tile, LDS_AS const float* scales, int t, int n_valid,
                        LDS_AS unsigned char* vtile, i32x8& P, int& sb, bool& jumped) {
        constexpr bool CAREFUL = decltype(careful_tag)::value;
        constexpr int OPH = 2 * NJ + 2;                      // operands per half
        constexpr int NO = 2 * OPH;                          // operands of the tile
        constexpr int D = 3;                                 // operands requested ahead (about 200 cycles of instructions)
        static_assert(OPH >= 6 && NO >= 2 * VP, "half 0's arithmetic and the first value reads ride on half 1's operands");
        static_assert(WCT >= 8, "half 1's arithmetic rides on the column tiles of the value contraction");
        f32x4 sacc[2][2], rs[2][2], rw[2][2];   // rs: the row scales as read for (2); rw: read again for (4) (not kept in between)
        u32x4 op[NO][2], qrv[2][2];   // qrv: the rope part of the query operand, read per half
        u32x2 vv[WCT][2];
        float x[2][2][4], w[16], wmax = 0.f, lsum = 0.f, f = 1.f, m_use = 0.f;
        i32x8 Pn;
        int sbn = ONE;
#pragma unroll
        for (int h = 0; h < 2; ++h) sacc[h][0] = sacc[h][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
        // (the lane's operand addresses are worked out per tile, each set where its reads begin, from
        // a lane index the compiler cannot see through: kept across the tile loop they cost registers
        // that the loop does not have)
        uint32_t ab[2], arb[2], vb[4];
        {
            int lane_o = lane;
            asm volatile("" : "+v"(lane_o));
            const int n = lane_o & 15, g = lane_o >> 4;
            const uint32_t row = (uint32_t)((8 * (n >> 2) + (n & 3)) * ROWB), key = (uint32_t)((n >> 2) & 1);   // block 0; block 1: 4 rows further, same key
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                ab[e] = row + (uint32_t)((g >> 1) * 64) + ((((uint32_t)((2 * g + e) & 3)) ^ key) << 4);
                arb[e] = row + (uint32_t)D_C + ((((uint32_t)(2 * (g & 1) + e)) ^ key) << 4);
            }
        }
        auto value_addresses = [&]() {
            int lane_o = lane;
            asm volatile("" : "+v"(lane_o));
            const int n = lane_o & 15, g = lane_o >> 4;
            const uint32_t base = (uint32_t)((8 * g + (n >> 1)) * ROWB + (n & 1) * 8), key = (uint32_t)(g & 1);
#pragma unroll
            for (int e = 0; e < 4; ++e) vb[e] = base + ((((uint32_t)e) ^ key) << 4);
        };
        auto ord = [&](int m) {
            const int h = m / OPH, r = m % OPH;
            LDS_AS unsigned char* half = tile + h * 32 * ROWB;
#pragma unroll
            for (int e = 0; e < 2; ++e)
                op[m][e] = r < 2 * NJ ? *(LDS_AS u32x4*)(half + ab[e] + (r & 1) * 4 * ROWB + (r >> 1) * A_STEP)
                                      : *(LDS_AS u32x4*)(half + arb[e] + (r - 2 * NJ) * 4 * ROWB);
        };
        auto finish = [&](int h) {   // (2) for half h
            const float unit = sc * q_unit;
            const int r0 = h * 32 + 8 * g;   // tile row behind D row 4g of block 0; block 1: 4 rows further
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int i = 0; i < 4; ++i) x[h][b][i] = sacc[h][b][i] * (unit * rs[h][b][i]);
            if (n_valid < TR || (t + 1) * TR > causal_from) {
                const int seen = min(n_valid, visible_rows(p, L, hb + head) - t * TR);
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (r0 + 4 * b + i >= seen) x[h][b][i] = -INFINITY;
            }
            reference_step(careful_tag, x[h][0], x[h][1], jumped);
            m_use = m_run == -INFINITY ? 0.f : m_run;   // only while every row so far is masked
        };
        auto take = [&](int e) {     // (4), element e = (half, block, i): the plain weight and the scaled one
            const float ex = fast_exp2(x[e >> 3][(e >> 2) & 1][e & 3] - m_use);
            lsum += ex;
            w[e] = ex * rw[e >> 3][(e >> 2) & 1][e & 3];
            wmax = fmaxf(wmax, w[e]);
            asm volatile("" : "+v"(w[e]));   // (keeps the arithmetic behind the instruction it is written behind)
        };
        auto scales_read = [&](int h, f32x4 (&r)[2][2]) {   // lane (g, n): rows 8g .. 8g+7 of half h
#pragma unroll
            for (int b = 0; b < 2; ++b) r[h][b] = *(LDS_AS const f32x4*)(scales + h * 32 + 8 * g + 4 * b);
        };
        auto scale = [&]() {         // (4), the pair's c
            // largest weight of the pair of lane groups (rows of 16 lanes: 0 with 1, 2 with 3)
            const u32x2 sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(wmax), __float_as_uint(wmax), false, false);
            wmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
            const int c = min(134 - (int)(__float_as_uint(wmax) >> 23), 127);
            f = __uint_as_float((uint32_t)(c + 127) << 23);              // 2^c (c >= -121)
            const uint32_t sb_pair = (uint32_t)(127 - c) * 0x01010101u;   // 2^-c as an e8m0 block scale, in every byte
            // halves of 32 lanes swapped: first result = pair 0's in every lane group, second = pair 1's
            const u32x2 ss = __builtin_amdgcn_permlane32_swap(sb_pair, sb_pair, false, false);
            sbn = (int)((g & 1) ? ss[1] : ss[0]);
        };
        auto convert = [&](int pr) { // (4), pair pr = (half, block): four weights -> one register of codes per term
            const float v0 = w[4 * pr] * f, v1 = w[4 * pr + 1] * f, v2 = w[4 * pr + 2] * f, v3 = w[4 * pr + 3] * f;
            int hi = __builtin_amdgcn_cvt_pk_fp8_f32(v0, v1, 0, false);
            hi = __builtin_amdgcn_cvt_pk_fp8_f32(v2, v3, hi, true);
            const f32x2 b01 = __builtin_amdgcn_cvt_pk_f32_fp8(hi, false);
            const f32x2 b23 = __builtin_amdgcn_cvt_pk_f32_fp8(hi, true);
            int lo = __builtin_amdgcn_cvt_pk_fp8_f32(v0 - b01[0], v1 - b01[1], 0, false);
            lo = __builtin_amdgcn_cvt_pk_fp8_f32(v2 - b23[0], v3 - b23[1], lo, true);
            Pn[pr] = hi;
            Pn[4 + pr] = lo;
        };

        // ---- (1), in the fast pass with half 0's (2) and (4) behind half 1's operands
#pragma unroll
        for (int m = 0; m < D; ++m) ord(m);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NO; ++m) {
            const int h = m / OPH, r = m % OPH;
            if (m + D < NO) ord(m + D);
            if (r == 2 * NJ - D) {   // with the half's first rope operand
                qrv[h][0] = qr_lds[w4][0][lane];
                qrv[h][1] = qr_lds[w4][1][lane];
            }
            if (m == NO - 2 * VP) value_addresses();
            if (m >= NO - 2 * VP && ((m - (NO - 2 * VP)) & 1) == 0)
                value_read(vtile, vb, (m - (NO - 2 * VP)) >> 1, vv[(m - (NO - 2 * VP)) >> 1]);
            const i32x8 k = __builtin_bit_cast(i32x8, __builtin_shufflevector(op[m][0], op[m][1], 0, 1, 2, 3, 4, 5, 6, 7));
            if (r < 2 * NJ) {
                sacc[h][r & 1] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(k, qhi[r >> 1], sacc[h][r & 1], 0, 0, 0, ONE, 0, ONE);
                sacc[h][r & 1] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(k, qlo[r >> 1], sacc[h][r & 1], 0, 0, 0, ONE, 0, ONE);
            } else {
                const i32x8 qr = __builtin_bit_cast(i32x8, __builtin_shufflevector(qrv[h][0], qrv[h][1], 0, 1, 2, 3, 4, 5, 6, 7));
                sacc[h][r - 2 * NJ] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(k, qr, sacc[h][r - 2 * NJ], 0, 0, 0, ONE, 0, ONE);
            }
            asm volatile("" : "+v"(sacc[h][r < 2 * NJ ? (r & 1) : r - 2 * NJ]) :: "memory");   // (as above)
            if (m == OPH - 3) scales_read(0, rs);
            if (m == NO - 3) scales_read(1, rs);
            if constexpr (!CAREFUL) {
                if (m == OPH - 1) scales_read(0, rw);
                if (m == OPH + 1) finish(0);
                if (m >= OPH + 2 && m < OPH + 6) { take(2 * (m - OPH - 2)); take(2 * (m - OPH - 2) + 1); }
                if (m == NO - 1) scales_read(1, rw);
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        if constexpr (CAREFUL) {
            // ---- (3), then (2) and (4), one after the other
#pragma unroll
            for (int i = 0; i < WCT; ++i) { value_step(vtile, vb, i, vv, P, sb); __builtin_amdgcn_sched_barrier(0); }
            scales_read(0, rw);
            scales_read(1, rw);
            finish(0);
#pragma unroll
            for (int e = 0; e < 8; ++e) take(e);
            finish(1);
#pragma unroll
            for (int e = 8; e < 16; ++e) take(e);
            scale();
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) convert(pr);
        } else {
            // ---- (2) of half 1, then (3) with half 1's (4) behind its column tiles
            finish(1);
#pragma unroll
            for (int i = 0; i < WCT; ++i) {
                value_step(vtile, vb, i, vv, P, sb);
                if (i < 4) { take(8 + 2 * i); take(8 + 2 * i + 1); }
                else if (i == 4) scale();
                else if (i < 7) convert(i - 5);
                else if (i == 7) { convert(2); convert(3); }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        l_run += lsum;
        P = Pn;
        sb = sbn;
    };

    // ---- one pass over the chunk's tiles.  CAREFUL = false: the fast pass, every head keeps the
    // maximum of its first tile with a visible row as the reference of all its exponentials and
    // only records whether a later score exceeded it by more than FAST_GAP.  CAREFUL = true: the
    // reference moves (and the accumulators are rescaled) whenever a tile maximum exceeds it by
    // more than RESCALE_GAP.  Producers and consumers execute the same barriers.
    int first_ahead = 0;   // producers: loads issued for the second tile of a pass by its first requests (below)
    auto sweep = [&](auto careful_tag) -> bool {
        constexpr bool CAREFUL = decltype(careful_tag)::value;
        static_assert(LOOK == 2, "the first requests (outside) cover the first tile and the one after it");
        int ahead[LOOK];       // producers: loads issued for the tiles after the one being consumed, oldest first
        ahead[0] = first_ahead;
        ahead[1] = 0;
        bool jumped = false;
        // fp8 consumers: the tile whose weights are ready and whose value contraction is still to come.
        // Before the first tile that is the first tile itself with weights zero (one contraction that
        // adds nothing, in exchange for a loop body without a case distinction: with one the
        // compiler keeps two copies of the accumulators).
        LDS_AS unsigned char* prev_tile = lds;
        i32x8 P_prev = {};
        int sb_prev = ONE;
        for (int t = t0; t < t1; ++t) {
            LDS_AS unsigned char* tile = lds + ((t - t0) % RING) * TILE_B;
            const int n_valid = rows_valid(t);
            if (producer) {
                // wait until my loads of tile t have landed (younger tiles may stay in flight)
                int younger = 0;
#pragma unroll
                for (int i = 0; i < LOOK; ++i) younger += ahead[i];
                wait_younger(younger);
            }
            // tile t has landed (every producer's part), and every consumer is done with tile t - 1
            __syncthreads();
            if (producer) {
                const int tn = t + LOOK;                 // goes into the slot tile t - 1 (fp8: t - 2) has left
                ahead[LOOK - 1] = tn < t1 ? fetch_tile(tn) : 0;
#pragma unroll
                for (int i = 0; i < LOOK - 1; ++i) ahead[i] = ahead[i + 1];   // tile t + 1 becomes the oldest in flight
                ahead[LOOK - 1] = 0;
            }
            if (n_valid < TR) {
                // ragged last tile (or a page id outside the pool): rows that are not part of the
                // sequence become zeros (fp8: and so do their scales) so that whatever they hold stays out
                for (int i = tid; i < (TR - n_valid) * CPR; i += ST_THREADS)
                    *(LDS_AS u32x4*)(tile + n_valid * ROWB + i * 16) = (u32x4){0u, 0u, 0u, 0u};
                if constexpr (FP8) {
                    if (tid >= n_valid && tid < TR) sc_lds[(t - t0) % RING][tid] = 0.f;
                }
                __syncthreads();
            }
            if (!producer) {
                LDS_AS const float* scales = (LDS_AS const float*)&sc_lds[FP8 ? (t - t0) % RING : 0][0];
                if constexpr (FP8) {
                    fp8_tile(careful_tag, tile, scales, t, n_valid, prev_tile, P_prev, sb_prev, jumped);
                    prev_tile = tile;
                } else {
                    float x0[4], x1[4], rs0[4], rs1[4];
                    f32x4 sacc0 = (f32x4){0.f, 0.f, 0.f, 0.f}, sacc1 = (f32x4){0.f, 0.f, 0.f, 0.f};
                    score_bf16(tile, sacc0, sacc1);
                    finish_scores(sacc0, sacc1, scales, t, 0, n_valid, x0, x1, rs0, rs1);
                    reference_step(careful_tag, x0, x1, jumped);
                    value_bf16(tile, weights(x0, x1));
                }
            }
        }
        if constexpr (FP8) {
            // the last tile's value contraction (consumers of a non-empty chunk always have one pending)
            if (!producer) {
                u32x2 vv[WCT][2];
                uint32_t vb[4];
                const uint32_t base = (uint32_t)((8 * g + (n >> 1)) * ROWB + (n & 1) * 8), key = (uint32_t)(g & 1);
#pragma unroll
                for (int e = 0; e < 4; ++e) vb[e] = base + ((((uint32_t)e) ^ key) << 4);
#pragma unroll
                for (int i = 0; i < VP; ++i) value_read(prev_tile, vb, i, vv[i]);
#pragma unroll
                for (int i = 0; i < WCT; ++i) { value_step(prev_tile, vb, i, vv, P_prev, sb_prev); __builtin_amdgcn_sched_barrier(0); }
            }
        }
        return jumped;
    };

    // ---- the first requests of a pass: (the query rows,) the first tile and the one after it.
    // Returns the number of loads this wave issued for the first tile; first_ahead = for the second.
    auto request_first = [&](bool with_query_rows) -> int {
        if (!producer) return 0;
        if (with_query_rows) fetch_query_rows();   // the oldest loads: every later wait covers them
        const int n0 = fetch_tile(t0);
        first_ahead = t0 + 1 < t1 ? fetch_tile(t0 + 1) : 0;
        return n0;
    };

    // ---- the query rows: requested first, awaited on their own (the tiles behind them stay in flight),
    // read by the consumers behind a barrier of their own.  (Inside the tile loop this one-time
    // code, which needs many registers, made the compiler spill accumulators in every iteration.)
    {
        const int n0 = request_first(true);
        if (producer) wait_younger(n0 + first_ahead);
        __syncthreads();
    }
    if (!producer) {
        // into registers, where they stay
        // (the addresses are derived here from a lane index the compiler cannot see through:
        // worked out ahead of the loop they would occupy registers all the way through it)
        int lane_q = lane;
        asm volatile("" : "+v"(lane_q));
        const int n = lane_q & 15, g = lane_q >> 4;
        const uint32_t q_row = (uint32_t)((hg * 16 + n) * QROWB);
        const uint32_t q_key = (uint32_t)swz_key(n);
        auto q_chunk = [&](int c) -> u32x4 {   // elements 8c .. 8c+7 of this lane's query row
            return *(LDS_AS u32x4*)(qlds + q_row + ((((uint32_t)c) ^ q_key) << 4));
        };
        if constexpr (FP8) {
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
#pragma unroll
            for (int c = 0; c < 4 * NJ; ++c) {
                int hi[2], lo[2];
                split8(q_chunk(16 * (c >> 2) + 4 * g + (c & 3)), hi, lo);
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    qhi[c >> 2][2 * (c & 3) + k] = hi[k];
                    qlo[c >> 2][2 * (c & 3) + k] = lo[k];
                }
            }
            i32x8 qr;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                int hi[2], lo[2];
                split8(q_chunk(D_C / 8 + 4 * (g & 1) + c), hi, lo);
#pragma unroll
                for (int k = 0; k < 2; ++k) qr[2 * c + k] = g < 2 ? hi[k] : lo[k];
            }
            // (read back by this wavefront only: its own LDS accesses complete in order)
            qr_lds[w4][0][lane_q] = (u32x4){(uint32_t)qr[0], (uint32_t)qr[1], (uint32_t)qr[2], (uint32_t)qr[3]};
            qr_lds[w4][1][lane_q] = (u32x4){(uint32_t)qr[4], (uint32_t)qr[5], (uint32_t)qr[6], (uint32_t)qr[7]};
        } else {
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                qreg[ks] = __builtin_bit_cast(bf16x8, q_chunk(4 * ks + g));
        }
    }

    const bool jumped = sweep(std::false_type{});
    if (jumped) jump_flag = 1;
    __syncthreads();   // every consumer is done with the last tile; nothing is in flight (the producers waited for it)
    if (__builtin_expect(jump_flag != 0, 0)) {
        // ---- careful pass (rare): the same chunk again with a moving reference
        m_run = -INFINITY;
        l_run = 0.f;
#pragma unroll
        for (int i = 0; i < WCT; ++i) oacc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
        request_first(false);
        sweep(std::true_type{});
        __syncthreads();
    }

    // ---- consumers: normalise and write the partial (bf16).  A consumer holds its column half of
    // its 16 heads complete; a lane holds 4 consecutive columns of head n per column tile, which
    // written straight out would give 8-byte pieces, so the block is transposed through LDS (the
    // tile ring is free: every wave has passed a barrier after its last tile) and stored in
    // whole runs of half a latent row.
    if (!producer) {
        float lt = l_run + __shfl_xor(l_run, 16);
        lt += __shfl_xor(lt, 32);
        const float inv = lt > 0.f ? 1.f / lt : 0.f;
        LDS_AS unsigned char* mine = lds + w4 * (16 * RSO);
#pragma unroll
        for (int i = 0; i < WCT; ++i) {
            const f32x4 o = oacc[i] * inv;
            *(LDS_AS u32x2*)(mine + n * RSO + (i * 16 + g * 4) * 2) =
                (u32x2){pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
        }
        const int nrow = min(16, HL - hg * 16);
        constexpr int LPR = WCT * 2;             // lanes (of 16 bytes = 8 bf16) covering one row of the half (32 / 16)
        constexpr int RPI = 64 / LPR;            // rows one store instruction covers (2 / 4)
        // all reads first, then all stores, from one base address and a row stride (computing the
        // address of every row anew, with a wait for its LDS read in between, tripled the time
        // of this loop)
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
            *lse_at(hb + head) = lt > 0.f ? (m_run + __builtin_amdgcn_logf(lt)) * LN2 : -INFINITY;
    }
    };  // run_segment

    // Workgroup -> (sequence, chunk): linear ids run over the sequences first, chunk by chunk, with
    // the sequence rotated by the chunk index (see decode_mfma.hip).
    const int cx = Z > 1 ? wg_lin % p.B : (int)blockIdx.x, cy = Z > 1 ? wg_lin / p.B : (int)blockIdx.y;
    run_segment((cx + cy) % p.B, cy, 0, 0, 0);
}

}  // namespace

hipError_t launch_decode_stream(const DecodeParams& p, dim3 grid, hipStream_t s, bool fp8)
{
    dim3 block(ST_THREADS);
    if (p.d_c == 512 && !fp8)      decode_stream_kernel<512, false><<<grid, block, 0, s>>>(p);
    else if (p.d_c == 256 && !fp8) decode_stream_kernel<256, false><<<grid, block, 0, s>>>(p);
    else if (p.d_c == 512 && fp8)  decode_stream_kernel<512, true><<<grid, block, 0, s>>>(p);
    else if (p.d_c == 256 && fp8)  decode_stream_kernel<256, true><<<grid, block, 0, s>>>(p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace mla
