// Matrix-core paged decode for a bf16 latent cache (gfx950 / CDNA4), and the dispatch of the other
// matrix-core decode kernels (decode_stream.hip, decode_stream_fp8.hip).  The kernel of this file
// serves d_c = 256 on long chunks and under the balanced partition (everything else at bf16 goes to
// decode_stream.hip's); the tile layout, the swizzle, the transposed formulation, the two passes
// and the balanced plan described here are shared by all of them.
//
// Second line of the absorbed attention equation (Sec. 3.3 of the paper): all
// H heads score against the ONE shared row k_hat_j = [c_j ; k^R_j] and weight
// the same latent rows c_j, so per tile of cached rows both contractions are
// dense:
//     S^T [tok x heads]   = K [tok x (d_c+64)] . Q^T [(d_c+64) x heads]
//     O^T [d_c x heads]  += V^T [d_c x tok] . P^T [tok x heads]
// with V = the first d_c columns of the very same LDS tile as K.
//
// Data movement.  The kernel is bound by streaming the cache from HBM, so the
// design goal is to keep as many bytes in flight per CU as LDS allows.  A tile
// is half a page (32 rows); a ring of four tiles fills LDS (4 x 36 KB at
// d_c = 512).  One tile is being consumed while up to three are in flight as
// direct-to-LDS 128-bit loads; a tile is requested the moment its ring slot is
// released.  Every row is fetched from HBM exactly once per workgroup and
// serves all heads.
//
// Work decomposition (workgroup = 4 wavefronts per (chunk, sequence)):
//   wave = (hg, tg): head group hg (16 heads) x row half tg (16 of the 32 rows).
//   Each wave runs a complete private online softmax for its 16 heads over its
//   own rows, so the only workgroup barrier per tile is the one that publishes
//   the tile; the two row halves are merged once at the end.
//
// Operand layouts (lane = 16*g + n):
//   v_mfma_f32_16x16x32_bf16: A = row n, k = 8g..8g+7; B = column n, k = 8g..8g+7
//   v_mfma_f32_16x16x16_bf16: A = row n, k = 4g..4g+3; B = column n, k = 4g..4g+3
//   both:                     D = rows 4g..4g+3 of column n.
// Transposed formulation: S^T puts heads on the D columns, so every lane owns ONE
// head: the row maximum needs two cross-lane steps, the rescale factor is a
// per-lane scalar, and the exponentiated scores (rows 4g..4g+3) are, as they
// stand, the B operand of the second contraction.  Its A operand V^T (four
// consecutive rows of one column per lane) comes from ds_read_b64_tr_b16, which
// transposes 4x16 blocks of 16-bit elements while reading LDS.
//
// LDS layout: row r of a tile occupies bytes [r*ROWB, (r+1)*ROWB); inside a row,
// 16-byte chunk c is stored at chunk position c ^ key(r), key(r) = r & 6 (see swz_key for
// the bank rule it answers).  ROWB is 128 bytes mod 256, so row parity picks the half of the
// 256-byte bank window and the key spreads the rest: the row-wise 128-bit reads of the score
// contraction run conflict-free, and a transposing read (4 rows x 32 bytes per 16 lanes) covers
// 16 different 8-byte units.
#include "mla_internal.h"
#include "mfma_tile.h"
#include <type_traits>

namespace mla {
namespace {

// bf16 caches (tiles go HBM -> LDS directly); fp8 caches have a kernel of their own
// (decode_stream_fp8.hip).
// NBUF = tiles in the LDS ring: 4 fills LDS with one workgroup per CU; 2 leaves room
//        for two workgroups per CU (WPE = waves per SIMD the register budget is sized for).
// BAL  = false: one workgroup per (sequence, chunk), chunks of the same number of pages.
//        true : the page lists of all sequences, laid end to end, are cut into as many equal
//               ranges as there are workgroups; a workgroup walks its range sequence by sequence
//               (one segment each) and writes one partial result per segment.
template <int D_C, int NBUF, int WPE, bool BAL>
__global__ __launch_bounds__(MF_THREADS, WPE) void decode_mfma_kernel(DecodeParams p)
{
    constexpr int ROW = D_C + 64;               // elements per cache row
    constexpr int ROWB = ROW * 2;               // bytes per row
    constexpr int CPR = ROWB / 16;              // 16-byte chunks per row (72 / 40)
    constexpr int PAGE_B = 64 * ROWB;           // bytes per page
    constexpr int TILE_B = TILE_ROWS * ROWB;    // bytes per tile
    constexpr int NLOAD = TILE_B / (MF_THREADS * 16);  // 16-byte loads per thread per tile (9 / 5)
    constexpr int NKS = ROW / 32;               // k-steps of the score contraction (18 / 10)
    constexpr int NCT = D_C / 16;               // column tiles of the value contraction (32 / 16)
    constexpr int SG = NKS % 3 == 0 ? 3 : 2;    // k-steps per read-ahead group (score)
    constexpr int VG = 8;                       // column tiles per read-ahead group (value)
    static_assert(TILE_B % (MF_THREADS * 16) == 0, "tile must split evenly over the loads");
    static_assert(CPR % 8 == 0, "chunk swizzle needs rows of whole 128-byte groups");
    static_assert(NLOAD * NBUF < 64, "vmcnt is a 6-bit counter");
    static_assert(NBUF >= 2 && NBUF <= 4, "ring depth");

    __shared__ __attribute__((aligned(1024))) unsigned char smem[NBUF * TILE_B];
    __shared__ int seg_lds[BAL ? 64 : 1][3];         // balanced partition: (sequence, first row, end row) per segment
    __shared__ int jump_flag;                        // raised by a wavefront whose fast pass met a score far above its reference
    LDS_AS unsigned char* lds = (LDS_AS unsigned char*)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hg = wave & 1, tg = wave >> 1;
    const int n = lane & 15, g = lane >> 4;
    // One segment = cached rows [row0, row1) of sequence b, reduced to one partial result.
    // BAL = false: the rows are those of chunk `split` of the sequence (seg_row0/1 unused) and the
    // result goes to partial (b, split); BAL = true: the caller gives the rows and the partial slot.
    // Query rows beyond 32 (several query tokens per sequence, or more than 32 heads) go to
    // further workgroups: this one takes rows [hb, hb + 32) of every sequence.  The grid is then
    // one-dimensional and the workgroups that share a chunk of cached rows get linear ids 8 apart:
    // ids are dealt round-robin to the 8 XCDs, so they run at the same time on CUs of one XCD and
    // all but the first find the rows in that XCD's L2.
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
    // Balanced partition: the body runs in a loop.  Everything derived from the thread index is
    // derived again here from a value the compiler cannot see through, so that none of it is
    // hoisted out of that loop and kept in registers across the epilogue (which has none to spare).
    int opaque_zero = 0;
    if constexpr (BAL) asm volatile("" : "+v"(opaque_zero));
    const int tid = (int)threadIdx.x + opaque_zero;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hg = wave & 1, tg = wave >> 1;
    const int n = lane & 15, g = lane >> 4;
    const int HL = min(32, p.H - hb);          // query rows of this workgroup
    // cleared here, read after the tile loop: at least one workgroup barrier lies between (every
    // chunk that reaches the loop stages a tile), and between one segment's read and the next
    // segment's clear (the barrier after run_segment)
    if (tid == 0) jump_flag = 0;
    // where query row h's (h counted over the whole sequence) partial row and log-sum-exp go
    auto o_row = [&](int h) -> uint16_t* {    // partial rows are bf16 (the io dtype of this kernel)
        return static_cast<uint16_t*>(p.o_part) + (BAL ? (out_slot * p.H + h) : part_index(b, h, split, p.H, p.num_splits)) * D_C;
    };
    auto lse_at = [&](int h) -> float* {
        return p.lse_part + (BAL ? (out_slot * p.H + h) : part_index(b, h, split, p.H, p.num_splits));
    };

    // Read-only tables go through the scalar cache: scalar loads do not count against the
    // vector-memory counter, so looking up a page id never waits on an in-flight prefetch.
    const CONST_AS int32_t* seq_lens_c = (const CONST_AS int32_t*)p.seq_lens;
    const CONST_AS int32_t* ptab = (const CONST_AS int32_t*)(p.page_table + (size_t)b * p.max_pages);
    // touch this chunk's first page-table line now, in parallel with the sequence length
    // (both are scalar loads): the later look-ups then hit the scalar cache
    const int warm = ptab[min(BAL ? seg_row0 / 64 : split * p.chunk_pages, p.max_pages - 1)];
    int L = seq_lens_c[b];

    // ---- this wave's 16 query rows as B operands, resident for the whole chunk: lane (g, n) holds
    // elements 8g .. 8g+7 of every 32-element k-step of head 16 hg + n.  They are requested here,
    // while the two scalar loads above are still on their way and ahead of the first tiles.
    // bf16 path: the loads are inline assembly like the tile loads, because the compiler, which
    // cannot see those, would otherwise wait for "everything in flight" (the whole ring) at the
    // first use of a query register; their arrival is awaited by count below, where the registers
    // are handed to the compiler.  (An earlier version sent the query rows through the last ring
    // slot: that slot could then not be requested before the rows had been copied to registers,
    // which left the memory system without requests for about 1.5 us at the start.)
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    const int head = hg * 16 + n;
    u32x4 qraw[NKS];
    {
        const int hq = min(head, HL - 1);     // absent heads read a present one; their registers are cleared below
        const uint16_t* qa = static_cast<const uint16_t*>(p.q_abs) + ((size_t)b * p.H + hb + hq) * D_C + g * 8;
        const uint16_t* qr = static_cast<const uint16_t*>(p.q_rope) + ((size_t)b * p.H + hb + hq) * 64 + g * 8;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const uint16_t* src = ks < D_C / 32 ? qa + ks * 32 : qr + (ks - D_C / 32) * 32;
            asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(qraw[ks]) : "v"(src) : "memory");
        }
    }

    asm volatile("" :: "s"(warm));
    L = max(0, min(L, p.max_pages * 64));
    const int row0 = BAL ? seg_row0 : split * p.chunk_pages * 64;             // first cached row of this segment
    const int row1 = BAL ? min(seg_row1, L) : min(row0 + p.chunk_pages * 64, L);  // one past its last row
    if (row0 >= row1) {  // empty chunk: weight zero in the merge, partial output never read
        if (tid < HL) *lse_at(hb + tid) = -INFINITY;
        wait_vmcnt<0>();  // the workgroup's LDS must not be released with loads into it in flight
        return;
    }
    const int t0 = row0 / TILE_ROWS;                                // tiles [t0, t1) of the sequence
    const int t1 = (row1 + TILE_ROWS - 1) / TILE_ROWS;

    bf16x8 qreg[NKS];

    // ---- tile staging: HBM -> LDS with direct-to-LDS 128-bit loads.
    // Load k of wave w fills LDS chunks [(4k+w)*64, +64) of the tile (the hardware writes lane
    // i at base + 16 i); LDS chunk P = row r, position pc holds the row's chunk
    // pc ^ key(r), so a wave still reads whole 128-byte lines from HBM.  The loads are
    // written as inline assembly on purpose: the compiler then keeps no record of pending LDS
    // writes and does not make LDS reads of the other ring slots wait for them.  Completion is
    // awaited explicitly (vmcnt) before the barrier that publishes a tile.
    uint32_t goff[NLOAD];   // byte offset of this thread's chunk inside a tile's rows
#pragma unroll
    for (int k = 0; k < NLOAD; ++k) {
        int P = (k * 4 + wave) * 64 + lane;
        int r = P / CPR, pc = P % CPR;
        goff[k] = (uint32_t)(r * ROWB + ((pc ^ swz_key(r)) << 4));
    }
    const unsigned char* kv = static_cast<const unsigned char*>(p.kv);

    // rows of tile t that belong to this chunk (0 if its page id is outside the pool)
    auto rows_valid = [&](int t) {
        int page = ptab[t >> 1];
        return (page >= 0 && page < p.num_pages) ? min(TILE_ROWS, row1 - t * TILE_ROWS) : 0;
    };
    // returns the number of loads this thread issued (0 or NLOAD; uniform)
    auto fetch_tile = [&](int t) -> int {
        if (rows_valid(t) <= 0) return 0;   // a page outside the pool is never dereferenced
        const unsigned char* src = kv + (size_t)ptab[t >> 1] * PAGE_B + (size_t)(t & 1) * TILE_B;
        const uint32_t dst = lds_base + (uint32_t)(((t - t0) % NBUF) * TILE_B + wave * 1024);
        if (stream_once) {
            // this workgroup is the only reader of these rows: non-temporal loads (measured on a
            // bare ring of the same loads: 6.7 instead of 6.0 TB/s over the chip)
#pragma unroll
            for (int k = 0; k < NLOAD; ++k) {
                const unsigned char* gp = src + goff[k];
                const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst + k * 4096);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
                             :: "s"(m0v), "v"(gp) : "memory");
            }
        } else {
            // further groups of query rows read the same rows from this XCD's L2: ordinary loads
#pragma unroll
            for (int k = 0; k < NLOAD; ++k) {
                const unsigned char* gp = src + goff[k];
                const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst + k * 4096);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                             :: "s"(m0v), "v"(gp) : "memory");
            }
        }
        return NLOAD;
    };


    // ---- running softmax state: this lane's head = column n of the D tiles
    float m_run = -INFINITY;   // reference of the exponentials, scaled scores in log2 units
    float l_run = 0.f;         // this lane's share of the running sum (its 4 rows per tile)
    f32x4 oacc[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) oacc[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const float sc = p.scale * LOG2E;
    // LDS byte offsets that do not depend on the tile.  A swizzled chunk index splits into a
    // per-lane part (low 3 bits, xor-ed with the row key) and a compile-time part (high bits).
    // score A operand: row 16tg + n, chunk 4ks + g
    const uint32_t a_row = (uint32_t)((tg * 16 + n) * ROWB);
    const uint32_t a_key = (uint32_t)swz_key(n);
    uint32_t a_base[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) a_base[e] = a_row + ((((uint32_t)(4 * e + g)) ^ a_key) << 4);
    // value A operand (transposing read): the lane supplies row 16tg + 4g + (n>>2),
    // 8 bytes at element column 16ct + 4(n&3), i.e. chunk 2ct + ((n&3)>>1), half (n&1)
    const uint32_t v_row = (uint32_t)((tg * 16 + g * 4 + (n >> 2)) * ROWB);
    const uint32_t v_key = (uint32_t)swz_key(g * 4 + (n >> 2));
    uint32_t v_base[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        v_base[e] = v_row + ((((uint32_t)(2 * e) + (uint32_t)((n & 3) >> 1)) ^ v_key) << 4) + (uint32_t)((n & 1) * 8);

    // ---- one tile: publish it, score it, fold it into the running softmax, accumulate.
    // `ahead` holds the loads issued for the tiles after the one being consumed, oldest first.
    int ahead[NBUF - 1];

    int first_issued = 0;   // loads issued for tile t0 by the last start_ring()
    auto slot_of = [&](int t) { return (t - t0) % NBUF; };

    bool ring_full = false;   // tile t0 + NBUF - 1 has been requested ahead of the first stage step
    // request tile t0 + NBUF - 1 into the last ring slot before the first stage step (which
    // then must not request it again)
    auto fill_last_slot = [&]() {
        ahead[NBUF - 2] = t0 + NBUF - 1 < t1 ? fetch_tile(t0 + NBUF - 1) : 0;
        ring_full = true;
    };
    auto start_ring = [&](bool whole_ring) {
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i) ahead[i] = 0;
        first_issued = fetch_tile(t0);   // every chunk that gets here has at least one tile
#pragma unroll
        for (int i = 0; i < NBUF - 2; ++i)
            if (t0 + 1 + i < t1) ahead[i] = fetch_tile(t0 + 1 + i);
        ring_full = false;
        if (whole_ring) fill_last_slot();
    };

    // publish tile t (and keep the stream going); returns its number of valid rows
    auto stage_tile = [&](int t, LDS_AS unsigned char* tile) -> int {
        const int n_valid = rows_valid(t);
        // wait until my loads of tile t have landed (younger tiles may stay in flight);
        // after the barrier everybody's have, and every wave is done with tile t-1, whose
        // ring slot now receives tile t + NBUF - 1
        int younger = 0;
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i) younger += ahead[i];   // the last entry is 0 unless ring_full
        if (NBUF > 3 && younger >= 3 * NLOAD)      wait_vmcnt<3 * NLOAD>();
        else if (NBUF > 2 && younger >= 2 * NLOAD) wait_vmcnt<2 * NLOAD>();
        else if (younger >= NLOAD)                 wait_vmcnt<NLOAD>();
        else                                       wait_vmcnt<0>();
        __syncthreads();
        if (!ring_full) {
            const int tn = t + NBUF - 1;
            ahead[NBUF - 2] = tn < t1 ? fetch_tile(tn) : 0;
        }
        ring_full = false;
        if (n_valid < TILE_ROWS) {
            // ragged last tile (or a page id outside the pool): rows that are not part of
            // the sequence become zeros so that whatever they hold stays out
            for (int i = tid; i < (TILE_ROWS - n_valid) * CPR; i += MF_THREADS)
                *(LDS_AS u32x4*)(tile + n_valid * ROWB + i * 16) = (u32x4){0u, 0u, 0u, 0u};
            __syncthreads();
        }
        // tile t+1 becomes the oldest one in flight
#pragma unroll
        for (int i = 0; i < NBUF - 2; ++i) ahead[i] = ahead[i + 1];
        ahead[NBUF - 2] = 0;
        return n_valid;
    };


    // S^T = K . Q^T for this wave's 16 rows x 16 heads, scaled to log2 units, invalid rows at
    // -inf; returns the maximum over this lane's 4 rows of its head.  Operand reads run
    // one group of SG k-steps ahead of the MFMAs; the scheduling fences keep the compiler from
    // sinking the reads back next to their uses.
    // first cached row (of the sequence) that some query row of the sequence must not see
    const int causal_from = L - (p.q_len - 1);
    auto score_tile = [&](LDS_AS unsigned char* tile, int t, int n_valid, float (&x)[4]) -> float {
        f32x4 sacc = (f32x4){0.f, 0.f, 0.f, 0.f};
        bf16x8 a0[NKS];
#pragma unroll
        for (int ks = 0; ks < SG; ++ks)
            a0[ks] = *(LDS_AS bf16x8*)(tile + a_base[ks & 1] + (ks >> 1) * 128);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s0 = 0; s0 < NKS; s0 += SG) {
#pragma unroll
            for (int ks = s0 + SG; ks < s0 + 2 * SG && ks < NKS; ++ks)
                a0[ks] = *(LDS_AS bf16x8*)(tile + a_base[ks & 1] + (ks >> 1) * 128);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = s0; ks < s0 + SG && ks < NKS; ++ks)
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[ks], qreg[ks], sacc, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = sacc[i] * sc;
        if (n_valid < TILE_ROWS || (t + 1) * TILE_ROWS > causal_from) {
            // ragged last tile, and the upper limit of this lane's query row (Eq. "mqa": the sum
            // runs up to the query token's own position)
            const int seen = min(n_valid, visible_rows(p, L, hb + head) - t * TILE_ROWS);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (tg * 16 + g * 4 + i >= seen) x[i] = -INFINITY;
        }
        return fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
    };
    // maximum over the four lane groups (the wave's 16 tile rows), on every lane: two LDS round
    // trips, taken only where that maximum is needed
    auto over_groups = [&](float v) {
        v = fmaxf(v, __shfl_xor(v, 16));
        return fmaxf(v, __shfl_xor(v, 32));
    };

    // weights p = 2^(x - m_run) rounded to bf16 (the normaliser sums exactly the rounded
    // weights), then O^T += V^T . P^T with transposing reads one group of VG tiles ahead
    auto accumulate_tile = [&](LDS_AS unsigned char* tile, const float (&x)[4]) {
        const float m_use = m_run == -INFINITY ? 0.f : m_run;  // only while every row so far is masked
        const uint32_t p01 = pack_bf16x2(fast_exp2(x[0] - m_use), fast_exp2(x[1] - m_use));
        const uint32_t p23 = pack_bf16x2(fast_exp2(x[2] - m_use), fast_exp2(x[3] - m_use));
        // the normaliser sums exactly the rounded weights that get multiplied
        l_run += (bf16_bits_to_f32(p01 & 0xFFFFu) + bf16_bits_to_f32(p01 >> 16)) +
                 (bf16_bits_to_f32(p23 & 0xFFFFu) + bf16_bits_to_f32(p23 >> 16));
        const s16x4 pb = __builtin_bit_cast(s16x4, (u32x2){p01, p23});
        s16x4 va[NCT];
#pragma unroll
        for (int ct = 0; ct < VG; ++ct)
            va[ct] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (LDS_AS s16x4*)(tile + v_base[ct & 3] + (ct >> 2) * 128));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c0 = 0; c0 < NCT; c0 += VG) {
#pragma unroll
            for (int ct = c0 + VG; ct < c0 + 2 * VG && ct < NCT; ++ct)
                va[ct] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (LDS_AS s16x4*)(tile + v_base[ct & 3] + (ct >> 2) * 128));
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ct = c0; ct < c0 + VG && ct < NCT; ++ct)
                oacc[ct] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va[ct], pb, oacc[ct], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- fast pass.  A head takes the maximum of its first tile with a valid row as the
    // reference m_run of all its exponentials and never moves it, so the output accumulators
    // are only ever touched by MFMA (no rescaling, no register shuffling).  That is exact as
    // long as no later score exceeds the reference by more than FAST_GAP (log2 units): then
    // p <= 2^FAST_GAP and neither p, the normaliser nor the accumulators can overflow.  A
    // larger jump is only recorded here; the chunk is then recomputed by the careful pass.
    {
        start_ring(true);
        // wait for the query rows only: the tile loads requested after them stay in flight
        // (vector memory loads complete in the order they were issued)
        {
            int later = first_issued;   // tile t0
#pragma unroll
            for (int i = 0; i < NBUF - 1; ++i) later += ahead[i];
            if (NBUF > 3 && later >= 4 * NLOAD)      wait_vmcnt<4 * NLOAD>();
            else if (NBUF > 2 && later >= 3 * NLOAD) wait_vmcnt<3 * NLOAD>();
            else if (later >= 2 * NLOAD)             wait_vmcnt<2 * NLOAD>();
            else if (later >= NLOAD)                 wait_vmcnt<NLOAD>();
            else                                     wait_vmcnt<0>();
        }
        // from here on the registers hold the rows: this is where the compiler learns of them
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            asm volatile("" : "+v"(qraw[ks]));
            if (head >= HL) qraw[ks] = (u32x4){0u, 0u, 0u, 0u};
            qreg[ks] = __builtin_bit_cast(bf16x8, qraw[ks]);
        }
    }

    bool jumped = false;
    for (int t = t0; t < t1; ++t) {
        const int slot = slot_of(t);
        LDS_AS unsigned char* tile = lds + slot * TILE_B;
        const int n_valid = stage_tile(t, tile);
        float x[4];
        const float lmax = score_tile(tile, t, n_valid, x);
        if (__any(m_run == -INFINITY)) {       // first tile with a visible row (as a rule: the first tile)
            const float tmax = over_groups(lmax);
            if (m_run == -INFINITY) m_run = tmax;
        }
        jumped |= lmax > m_run + FAST_GAP;
        accumulate_tile(tile, x);
    }

    // a plain flag and one barrier: the library's workgroup-wide OR costs about 1400 cycles here,
    // at a point where no cached row is in flight any more
    if (jumped) jump_flag = 1;
    __syncthreads();
    if (__builtin_expect(jump_flag != 0, 0)) {
        // ---- careful pass (rare): the same chunk again with a moving reference.  The tile
        // loop is nested in an outer loop whose body rescales the accumulators; the inner loop
        // is left, before the offending tile is accumulated, whenever a tile maximum exceeds
        // the reference by more than RESCALE_GAP, and that tile is then scored again.
        m_run = -INFINITY;
        l_run = 0.f;
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) oacc[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
        start_ring(true);
        int t = t0;
        bool staged = false;       // tile t has already been through its stage step
        int n_valid = 0;
        float alpha = 1.f;         // pending rescale factor of this lane's head
        while (true) {
            if (__any(alpha != 1.f)) {
                l_run *= alpha;
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct) oacc[ct] *= alpha;
                alpha = 1.f;
            }
            bool rescale = false;
            for (; t < t1; ++t) {
                const int slot = slot_of(t);
                LDS_AS unsigned char* tile = lds + slot * TILE_B;
                if (!staged) n_valid = stage_tile(t, tile);
                staged = false;
                float x[4];
                const float tmax = over_groups(score_tile(tile, t, n_valid, x));
                if (m_run == -INFINITY) m_run = tmax;     // nothing accumulated yet: nothing to rescale
                if (__any(tmax > m_run + RESCALE_GAP)) {
                    const float m_new = tmax > m_run + RESCALE_GAP ? tmax : m_run;
                    alpha = fast_exp2(m_run - m_new);     // 1 for the lanes that keep their reference
                    m_run = m_new;
                    staged = true;
                    rescale = true;
                    break;
                }
                accumulate_tile(tile, x);
            }
            if (!rescale) break;
        }
        __syncthreads();  // every wave is done with the tiles of the second pass too
    }

    // ---- merge the two row halves of each head group, normalise, write the partial (bf16).
    // Both wavefronts of a head group hold all D_C columns for their 16 tile rows.  Each hands the
    // column half it does not finish to its partner through LDS, rounded to bf16 (the partial is
    // stored in bf16 anyway; this halves the LDS traffic of the epilogue, during which no
    // cached row is in flight), and finishes the other half: combine, transpose (a lane holds 4
    // consecutive columns of head n per column tile, which written straight out would give
    // 32-byte runs) and store whole 1 KB runs.
    float l_w = l_run + __shfl_xor(l_run, 16);
    l_w += __shfl_xor(l_w, 32);
    // Every wave has passed a barrier after its last tile read and nothing is in flight: the
    // tile ring is free and serves as exchange space.
    constexpr int HCT = NCT / 2;             // column tiles each wavefront finishes
    constexpr int RSO = HCT * 32 + 32;       // row stride of the transposed half in bytes (padded: conflict-free both ways)
    constexpr int XCH = (HCT * 512 + 512) > 16 * RSO ? (HCT * 512 + 512) : 16 * RSO;  // per wavefront
    static_assert(4 * XCH <= NBUF * TILE_B, "exchange space must fit in the tile ring");
    LDS_AS unsigned char* mine = lds + (hg * 2 + tg) * XCH;          // written by the partner
    LDS_AS unsigned char* theirs = lds + (hg * 2 + (tg ^ 1)) * XCH;  // written by this wavefront
    auto hand_over = [&](auto first) {
        constexpr int C0 = decltype(first)::value;
#pragma unroll
        for (int i = 0; i < HCT; ++i)
            *(LDS_AS u32x2*)(theirs + (i * 64 + lane) * 8) =
                (u32x2){pack_bf16x2(oacc[C0 + i][0], oacc[C0 + i][1]), pack_bf16x2(oacc[C0 + i][2], oacc[C0 + i][3])};
    };
    if (tg == 0) hand_over(std::integral_constant<int, HCT>{});
    else         hand_over(std::integral_constant<int, 0>{});
    *(LDS_AS float*)(theirs + HCT * 512 + lane * 4) = m_run;
    *(LDS_AS float*)(theirs + HCT * 512 + 256 + lane * 4) = l_w;
    __syncthreads();
    const float m1 = *(LDS_AS float*)(mine + HCT * 512 + lane * 4);
    const float l1 = *(LDS_AS float*)(mine + HCT * 512 + 256 + lane * 4);
    const float m_all = fmaxf(m_run, m1);
    const float m_use = m_all == -INFINITY ? 0.f : m_all;
    const float w0 = fast_exp2(m_run - m_use), w1 = fast_exp2(m1 - m_use);
    const float lt = l_w * w0 + l1 * w1;
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    const float s0 = w0 * inv, s1 = w1 * inv;
    // combine in registers first; this wavefront's area is then free and is reused for the
    // transposition (only this wavefront touches it now, and LDS executes a wavefront's
    // accesses in order)
    auto finish_half = [&](auto first) {
        constexpr int C0 = decltype(first)::value;
#pragma unroll
        for (int i = 0; i < HCT; ++i) {
            const u32x2 b1 = *(LDS_AS u32x2*)(mine + (i * 64 + lane) * 8);
            const f32x4 o1 = (f32x4){bf16_bits_to_f32(b1[0] & 0xFFFFu), __uint_as_float(b1[0] & 0xFFFF0000u),
                                     bf16_bits_to_f32(b1[1] & 0xFFFFu), __uint_as_float(b1[1] & 0xFFFF0000u)};
            oacc[C0 + i] = oacc[C0 + i] * s0 + o1 * s1;
        }
#pragma unroll
        for (int i = 0; i < HCT; ++i)
            *(LDS_AS u32x2*)(mine + n * RSO + (i * 16 + g * 4) * 2) =
                (u32x2){pack_bf16x2(oacc[C0 + i][0], oacc[C0 + i][1]), pack_bf16x2(oacc[C0 + i][2], oacc[C0 + i][3])};
    };
    if (tg == 0) finish_half(std::integral_constant<int, 0>{});
    else         finish_half(std::integral_constant<int, HCT>{});
    const int nrow = min(16, HL - hg * 16);
    constexpr int LPR = HCT * 2;             // lanes (of 16 bytes = 8 bf16) covering one row of the half
    constexpr int RPI = 64 / LPR;            // rows one store instruction covers (2 or 4)
    static_assert(LPR == 32 || LPR == 16, "half a latent row is 512 B or 256 B");
    // all reads first, then all stores, from one base address and a row stride (an address
    // computed anew for every row, with a wait for its LDS read in between, tripled this loop)
    {
        const size_t row_stride = (size_t)(BAL ? 1 : p.num_splits) * D_C;   // elements between the partial rows of consecutive heads
        const int rl = lane / LPR, c = lane % LPR;
        uint16_t* dst0 = o_row(hb + hg * 16) + (size_t)rl * row_stride + tg * (HCT * 16) + c * 8;
        u32x4 v[16 / RPI];
#pragma unroll
        for (int j = 0; j < 16 / RPI; ++j) v[j] = *(LDS_AS u32x4*)(mine + (j * RPI + rl) * RSO + c * 16);
#pragma unroll
        for (int j = 0; j < 16 / RPI; ++j)
            if (j * RPI + rl < nrow)
                __builtin_nontemporal_store(v[j], reinterpret_cast<u32x4*>(dst0 + (size_t)(j * RPI) * row_stride));
    }
    if (tg == 0 && head < HL && g == 0)
        *lse_at(hb + head) = lt > 0.f ? (m_all + __builtin_amdgcn_logf(lt)) * LN2 : -INFINITY;
    };  // run_segment

    if constexpr (!BAL) {
        // Workgroup -> (sequence, chunk).  Linear ids run over the sequences first, chunk by
        // chunk, with the sequence rotated by the chunk index.  Ids are dealt round-robin to the
        // 8 XCDs and, inside an XCD, to its CUs in a fixed order, so any regular pattern in the ids
        // repeats on the hardware: with the chunks of a sequence adjacent, the empty trailing
        // chunks of short sequences fell on the same CUs every time and left half the chip idle,
        // and a sequence's chunks all went to the XCDs of its low chunk indices.  This order puts
        // the empty chunks (high chunk indices) at the end of the grid and spreads every
        // sequence over the XCDs.
        const int cx = Z > 1 ? wg_lin % p.B : (int)blockIdx.x, cy = Z > 1 ? wg_lin / p.B : (int)blockIdx.y;
        run_segment((cx + cy) % p.B, cy, 0, 0, 0);
    } else {
        // ---- balanced partition.  Pages of sequence b: P_b = ceil(len_b / 64); workgroup w of G
        // owns the global pages [P w / G, P (w+1) / G) of the concatenation, P = sum_b P_b (the
        // host has checked that B * max_pages fits 31 bits).  Every wavefront derives the same
        // plan by itself: lanes stand for sequences (64 at a time), a wave scan gives each
        // sequence's first and last global page.  The segments of a block of 64 sequences are
        // written to a small list in LDS first, so that nothing but a few wave-uniform counters
        // stays live across the segment body (the kernel has no registers to spare).
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
                    // the plan for the merge: sequence bb's partials are the slots first ..
                    // first + cnt - 1 (slot of a segment = workgroup + sequence index: strictly
                    // increasing along the concatenation, so no two segments share one)
                    p.plan[2 * bb] = pg > 0 ? w0 + bb : 0;
                    p.plan[2 * bb + 1] = w1 - w0 + 1;
                }
                if (ps == pe && pg > 0 && wave == 0 && w0 <= wg && wg <= w1) {
                    // A workgroup with an empty range (more workgroups than pages) still owns a
                    // slot if it lies inside a sequence's span: mark it empty for the merge.
                    for (int h = 0; h < p.H; ++h) p.lse_part[((size_t)wg + bb) * p.H + h] = -INFINITY;
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

bool decode_mfma_supported(const DecodeParams& p, mla_dtype io, mla_dtype cache)
{
    return io == MLA_BF16 && (cache == MLA_BF16 || cache == MLA_FP8_E4M3) && p.page_size == 64 &&
           p.d_rope == 64 && (p.d_c == 256 || p.d_c == 512) && p.H >= 1 &&
           ((long long)p.B * p.num_splits + 7) / 8 * 8 * ((p.H + 31) / 32) <= 0x7FFFFFFFLL;
}

// one-dimensional grid: (sequence, chunk) pairs, padded to a multiple of 8, x groups of 32 query rows
static unsigned grid_1d(const DecodeParams& p)
{
    const long long n = (long long)p.B * p.num_splits, Z = (p.H + 31) / 32;
    return (unsigned)(Z > 1 ? (n + 7) / 8 * 8 * Z : n);
}

// Ring depth of the bf16 kernels.  The wavefronts that consume a tile are the ones that request the
// next: while they stand in the memory pipe's queue the rows they asked for earlier land, so at
// the end of a chunk NBUF - 1 tiles are still waiting to be consumed after the last request has
// gone out.  A short chunk (C2: 16 tiles) pays for every tile of that backlog and runs best with
// three slots (measured 30.2 -> 29.2 us; two slots leave the memory system without a request between
// tiles: 31.5 us); on long chunks the deeper ring is the faster one (C3: 202.7 against 206 us).
static int ring_depth(const DecodeParams& p, bool balanced)
{
    const long long tiles = balanced ? 2LL * p.max_pages / (p.num_splits > 0 ? p.num_splits : 1) : 2LL * p.chunk_pages;
    return tiles <= 64 ? 3 : 4;
}

template <int D_C, bool BAL>
static void launch_one(const DecodeParams& p, dim3 grid, dim3 block, hipStream_t s, int depth)
{
    if (depth == 3) decode_mfma_kernel<D_C, 3, 1, BAL><<<grid, block, 0, s>>>(p);
    else            decode_mfma_kernel<D_C, 4, 1, BAL><<<grid, block, 0, s>>>(p);
}

hipError_t launch_decode_mfma(const DecodeParams& p, mla_dtype cache, hipStream_t s, bool balanced)
{
    const bool fp8 = cache == MLA_FP8_E4M3;
    dim3 block(MF_THREADS);
    const int depth = ring_depth(p, balanced);
    if (balanced) {
        if (!p.plan) return hipErrorInvalidValue;
        // workgroups = sequences x chunks per sequence (x groups of 32 query rows)
        dim3 grid(grid_1d(p));
        if (fp8) return launch_decode_stream_fp8(p, grid, s, true);
        // d_c = 512: the two-stage kernel (C3: 202.3 against 204.7 us per launch)
        if (p.d_c == 512) return launch_decode_stream_balanced(p, grid, s);
        if (p.d_c == 256) launch_one<256, true>(p, grid, block, s, depth);
        else return hipErrorInvalidValue;
        return hipGetLastError();
    }
    dim3 grid(p.B, p.num_splits);
    if (p.H > 32) grid = dim3(grid_1d(p));
    // d_c = 512, and short chunks at d_c = 256: the kernel with requesting-and-scoring wavefronts apart
    // from the accumulating ones (C2: 29.0 -> 27.5 us; the C3 cache in 4 uniform chunks of up to 256
    // tiles: 280 -> 230 us).  On long chunks at d_c = 256 the two are level per launch and this
    // file's kernel is ahead per step (C4, 64 tiles: 52.9 against 53.0 us, 66.4 against 67.4 us)
    if (!fp8 && (p.d_c == 512 || 2LL * p.chunk_pages <= 32)) return launch_decode_stream(p, grid, s);
    // fp8 caches, either partition, any chunk length: the kernel that contracts the codes as they are
    // (C5: 92.4 -> 62 us against an fp8 variant of the kernel above that widened every tile to bf16 in
    // LDS before it was consumed; that variant is gone)
    if (fp8) return launch_decode_stream_fp8(p, grid, s, false);
    if (p.d_c == 256) launch_one<256, false>(p, grid, block, s, depth);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace mla
