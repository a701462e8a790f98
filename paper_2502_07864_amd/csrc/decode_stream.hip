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
// SIMD, and the work of a tile is cut in two stages that run one tile apart:
//   wavefronts 4..7 (producers) request the tiles (nine 128-bit direct-to-LDS loads per tile
//     each), wait for them by count, and SCORE: producer (hg, rb) holds the query rows of heads
//     16 hg .. 16 hg + 15 in registers and contracts 16-row block rb of tile t + 1 against them
//     while the consumers work on tile t; the scaled scores (one 128-bit value per lane) go
//     through a small double-buffered LDS array;
//   wavefronts 0..3 (consumers) never touch the vector-memory counter.  Consumer (hg, ch) owns
//     heads 16 hg .. 16 hg + 15 and latent columns [ch d_c/2, (ch+1) d_c/2) for ALL 32 rows of a
//     tile: it picks up both blocks' scores, forms the weights and accumulates its column half
//     with K = 32 (one v_mfma_f32_16x16x32_bf16 per column tile, fed by two transposing LDS
//     reads).  Its 64 accumulator registers hold complete sums, so the epilogue is normalise,
//     transpose, store: no hand-over, no combine.
// Neither kind needs a whole tile period for its share (about 0.7 and 0.55 of it at d_c = 512), so
// the sweep follows the memory stream also where the shader clock is at the low end of its range;
// with the scores on the consumers as well, those needed 0.8 to 0.85 of the period and set the
// pace there.  Both kinds meet at one workgroup barrier per tile (tile t's scores are written,
// tile t + 1 has landed, everybody is done with tile t - 1, whose slot the producers then fill
// again).
#include "mla_internal.h"
#include "mfma_tile.h"
#include <type_traits>

namespace mla {
namespace {

constexpr int ST_THREADS = 512;   // 4 consumer (weights, values) + 4 producer (requests, scores) wavefronts

typedef __attribute__((ext_vector_type(8))) short s16x8;

// PROBE = true: the diagnostic variant behind mla_diag_stream_tiles: the same tile requests, waits and
// barriers, no query rows, no arithmetic, no output (how fast this launch shape can stream at all).
// BAL = true: the balanced partition (one-dimensional grid; a workgroup owns an equal share of the
// pages of all sequences and works through the segments of sequences inside it, exactly as in
// decode_mfma.hip, whose plan and slot numbering this is).
template <int D_C, bool PROBE, bool BAL>
__global__ __launch_bounds__(ST_THREADS, 1) void decode_stream_kernel(DecodeParams p)
{
    constexpr int NBUF = 4;                     // ring slots: tile t (values), tile t + 1 (scores), two on their way
    constexpr int ROW = D_C + 64;               // elements per cache row
    constexpr int ROWB = ROW * 2;               // bytes per row
    constexpr int CPR = ROWB / 16;              // 16-byte chunks per row (72 / 40)
    constexpr int PAGE_B = 64 * ROWB;           // bytes per page
    constexpr int TILE_B = TILE_ROWS * ROWB;    // bytes per tile
    constexpr int NLOAD = TILE_B / (256 * 16);  // 16-byte loads per producer thread per tile (9 / 5)
    constexpr int NKS = ROW / 32;               // k-steps of the score contraction (18 / 10)
    constexpr int WCT = D_C / 32;               // column tiles of the value contraction per consumer (16 / 8)
    constexpr int SG = NKS % 3 == 0 ? 3 : 2;    // k-steps per read-ahead group (score)
    constexpr int VG = 4;                       // column tiles per read-ahead group (value)
    constexpr int RSO = WCT * 32 + 32;          // epilogue: row stride of the transposed block in bytes (padded)
    static_assert(TILE_B % (256 * 16) == 0, "tile must split evenly over the producers' loads");
    static_assert(CPR % 8 == 0, "chunk swizzle needs rows of whole 128-byte groups");
    static_assert(NLOAD * (NBUF + 1) < 64, "vmcnt is a 6-bit counter");
    static_assert(4 * 16 * RSO <= NBUF * TILE_B, "the epilogue's transposition space must fit in the tile ring");

    __shared__ __attribute__((aligned(1024))) unsigned char smem[NBUF * TILE_B];
    // (the query rows [q_abs | q_rope] of the 32 heads travel like a cache tile, one row per head with
    // the same chunk swizzle: requested as direct-to-LDS loads into the ring's last slot right after
    // the first tile, read into the producers' registers after the first barrier; then the slot
    // joins the ring)
    // scaled scores of a tile's two 16-row blocks, from the wavefronts that score to those that
    // accumulate: [tile parity][head group][block][lane]
    __shared__ f32x4 xbuf[2][2][2][64];
    __shared__ int jump_flag;                        // raised by a consumer whose fast pass met a score far above its reference
    __shared__ int seg_lds[BAL ? 64 : 1][3];         // balanced partition: this workgroup's segments within a block of 64 sequences
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

    // one chunk (uniform partition) or one segment (balanced: rows [seg_row0, seg_row1) of sequence b,
    // partials into slot out_slot)
    auto run_segment = [&](const int b, const int split, const int seg_row0, const int seg_row1,
                           const size_t out_slot) {
    // (balanced partition: everything derived from the thread index is derived again per segment
    // from a value the compiler cannot see through, so that it is not kept in registers across
    // segments)
    int opaque_zero = 0;
    if constexpr (BAL) asm volatile("" : "+v"(opaque_zero));
    const int tid = BAL ? (int)threadIdx.x + opaque_zero : (int)threadIdx.x;
    const int lane = BAL ? (tid & 63) : (int)(threadIdx.x & 63);
    const int wave = __builtin_amdgcn_readfirstlane(BAL ? tid >> 6 : (int)threadIdx.x >> 6);
    const bool producer = wave >= 4;
    const int w4 = wave & 3;
    const int hg = w4 & 1, ch = w4 >> 1;       // head group; consumers: column half, producers: 16-row block
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
    // A wavefront scores or accumulates for life, and one register allocation serves both kinds: the
    // query rows of the scoring wavefronts (B operands, resident for the whole chunk: lane (g, n) holds
    // elements 8g .. 8g+7 of every 32-element k-step of head 16 hg + n; 72 / 40 registers) and the
    // accumulators of the others (64 / 32) are therefore the SAME registers, st[]
    constexpr int NST = NKS > WCT ? NKS : WCT;
    f32x4 st[NST];

    asm volatile("" :: "s"(warm));
    L = max(0, min(L, p.max_pages * 64));
    const int row0 = BAL ? seg_row0 : split * p.chunk_pages * 64;                  // first cached row of this chunk
    const int row1 = BAL ? min(seg_row1, L) : min(row0 + p.chunk_pages * 64, L);   // one past its last row
    if (row0 >= row1) {  // empty chunk: weight zero in the merge, partial output never read
        if (!PROBE && tid < HL) *lse_at(hb + tid) = -INFINITY;
        return;
    }
    const int t0 = row0 / TILE_ROWS;                                // tiles [t0, t1) of the sequence
    const int t1 = (row1 + TILE_ROWS - 1) / TILE_ROWS;

    // rows of tile t that belong to this chunk (0 if its page id is outside the pool)
    auto rows_valid = [&](int t) {
        int page = ptab[t >> 1];
        return (page >= 0 && page < p.num_pages) ? min(TILE_ROWS, row1 - t * TILE_ROWS) : 0;
    };

    // ---- producers: tile staging, HBM -> LDS with direct-to-LDS 128-bit loads (inline assembly:
    // the compiler keeps no record of them).  Load k of producer w fills LDS chunks [(4k+w)*64, +64)
    // of the tile; LDS chunk P = row r, position pc holds the row's chunk pc ^ key(r).
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    uint32_t goff[NLOAD];   // byte offset of this thread's chunk inside a tile's rows
#pragma unroll
    for (int k = 0; k < NLOAD; ++k) {
        int P = (k * 4 + w4) * 64 + lane;
        int r = P / CPR, pc = P % CPR;
        goff[k] = (uint32_t)(r * ROWB + ((pc ^ swz_key(r)) << 4));
    }
    const unsigned char* kv = static_cast<const unsigned char*>(p.kv);
    // returns the number of loads this thread issued (0 or NLOAD; uniform)
    auto fetch_tile = [&](int t) -> int {
        if (rows_valid(t) <= 0) return 0;   // a page outside the pool is never dereferenced
        const unsigned char* src = kv + (size_t)ptab[t >> 1] * PAGE_B + (size_t)(t & 1) * TILE_B;
        const uint32_t dst = lds_base + (uint32_t)(((t - t0) % NBUF) * TILE_B + w4 * 1024);
        if (stream_once) {
            // this workgroup is the only reader of these rows: non-temporal loads
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
            const int r = P / CPR, c = (P % CPR) ^ swz_key(r);
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

    // ---- running softmax state (consumers); this lane's head = column n of the D tiles, its rows
    // 4g .. 4g+3 of each of the tile's two 16-row blocks
    float m_run = -INFINITY;   // reference of the exponentials, scaled scores in log2 units
    float l_run = 0.f;         // this lane's share of the running sum (its 8 rows per tile)
#pragma unroll
    for (int i = 0; i < NST; ++i) st[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const float sc = p.scale * LOG2E;
    // score A operand: row 16 rb + n, chunk 4 ks + g
    const uint32_t a_row = (uint32_t)(n * ROWB);
    const uint32_t a_key = (uint32_t)swz_key(n);
    uint32_t a_base[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) a_base[e] = a_row + ((((uint32_t)(4 * e + g)) ^ a_key) << 4);
    // value A operand (transposing reads): the lane supplies row 16 rb + 4g + (n>>2), 8 bytes at
    // element column 16 ct + 4 (n&3), i.e. chunk 2 ct + ((n&3)>>1), half (n&1)
    const uint32_t v_row = (uint32_t)((g * 4 + (n >> 2)) * ROWB);
    const uint32_t v_key = (uint32_t)swz_key(g * 4 + (n >> 2));
    uint32_t v_base[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        v_base[e] = v_row + ((((uint32_t)(2 * e) + (uint32_t)((n & 3) >> 1)) ^ v_key) << 4) + (uint32_t)((n & 1) * 8);
    // first cached row (of the sequence) that some query row of the sequence must not see
    const int causal_from = L - (p.q_len - 1);
    // maximum over the four lane groups (a block's 16 rows), on every lane
    auto over_groups = [&](float v) {
        v = fmaxf(v, __shfl_xor(v, 16));
        return fmaxf(v, __shfl_xor(v, 32));
    };

    // S^T = K . Q^T for 16-row block rb of a tile x 16 heads, scaled to log2 units, rows outside the
    // chunk or beyond the query row's own position at -inf
    auto score_block = [&](LDS_AS unsigned char* tile, int rb, int t, int n_valid, f32x4& x) {
        f32x4 sacc = (f32x4){0.f, 0.f, 0.f, 0.f};
        bf16x8 a0[NKS];
        LDS_AS unsigned char* rows = tile + rb * 16 * ROWB;
        auto rd = [&](int ks) { a0[ks] = *(LDS_AS bf16x8*)(rows + a_base[ks & 1] + (ks >> 1) * 128); };
#pragma unroll
        for (int ks = 0; ks < SG; ++ks) rd(ks);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s0 = 0; s0 < NKS; s0 += SG) {
#pragma unroll
            for (int ks = s0 + SG; ks < s0 + 2 * SG && ks < NKS; ++ks) rd(ks);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = s0; ks < s0 + SG && ks < NKS; ++ks)
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[ks], __builtin_bit_cast(bf16x8, st[ks]), sacc, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        x = sacc * sc;
        if (n_valid < TILE_ROWS || (t + 1) * TILE_ROWS > causal_from) {
            const int seen = min(n_valid, visible_rows(p, L, hb + head) - t * TILE_ROWS);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (rb * 16 + g * 4 + i >= seen) x[i] = -INFINITY;
        }
    };

    // weights p = 2^(x - m_run) rounded to bf16 (the normaliser sums exactly the rounded weights),
    // then O^T += V^T . P^T over the tile's 32 rows: k slot 8g + j of the second contraction is
    // tile row 4g + j (j < 4) or 16 + 4g + j - 4, which is how the weights lie in the registers
    // after scoring and what two transposing reads (one per 16-row block) deliver
    auto accumulate_tile = [&](LDS_AS unsigned char* tile, const f32x4 x0, const f32x4 x1) {
        const float m_use = m_run == -INFINITY ? 0.f : m_run;  // only while every row so far is masked
        const uint32_t p01 = pack_bf16x2(fast_exp2(x0[0] - m_use), fast_exp2(x0[1] - m_use));
        const uint32_t p23 = pack_bf16x2(fast_exp2(x0[2] - m_use), fast_exp2(x0[3] - m_use));
        const uint32_t p45 = pack_bf16x2(fast_exp2(x1[0] - m_use), fast_exp2(x1[1] - m_use));
        const uint32_t p67 = pack_bf16x2(fast_exp2(x1[2] - m_use), fast_exp2(x1[3] - m_use));
        l_run += ((bf16_bits_to_f32(p01 & 0xFFFFu) + bf16_bits_to_f32(p01 >> 16)) +
                  (bf16_bits_to_f32(p23 & 0xFFFFu) + bf16_bits_to_f32(p23 >> 16))) +
                 ((bf16_bits_to_f32(p45 & 0xFFFFu) + bf16_bits_to_f32(p45 >> 16)) +
                  (bf16_bits_to_f32(p67 & 0xFFFFu) + bf16_bits_to_f32(p67 >> 16)));
        const bf16x8 pb = __builtin_bit_cast(bf16x8, (u32x4){p01, p23, p45, p67});
        s16x4 lo[WCT], hi[WCT];
        auto rd = [&](int i) {
            const int ct = ch * WCT + i;
            LDS_AS unsigned char* a = tile + v_base[ct & 3] + (ct >> 2) * 128;
            lo[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)a);
            hi[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(a + 16 * ROWB));
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
            for (int i = c0; i < c0 + VG && i < WCT; ++i) {
                const s16x8 va = __builtin_shufflevector(lo[i], hi[i], 0, 1, 2, 3, 4, 5, 6, 7);
                st[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, va), pb, st[i], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- one pass over the chunk's tiles.  CAREFUL = false: the fast pass, every head keeps the
    // maximum of its first tile with a visible row as the reference of all its exponentials and
    // only records whether a later score exceeded it by more than FAST_GAP.  CAREFUL = true: the
    // reference moves (and the accumulators are rescaled) whenever a tile maximum exceeds it by
    // more than RESCALE_GAP.  Producers and consumers execute the same barriers.
    auto sweep = [&](auto careful_tag) -> bool {
        constexpr bool CAREFUL = decltype(careful_tag)::value;
        // the query rows travel in slot 3, which joins the ring when the scoring wavefronts have read them
        constexpr bool Q_IN_RING = !CAREFUL && !PROBE;
        const int rb = ch;   // producers: the 16-row block of every tile this wavefront scores (for head group hg)
        auto await_all_but = [&](int younger) {
            if (younger >= 2 * NLOAD)  wait_vmcnt<2 * NLOAD>();
            else if (younger >= NLOAD) wait_vmcnt<NLOAD>();
            else                       wait_vmcnt<0>();
        };
        int c3 = 0;   // producers: loads issued for tile t0 + 3
        {
            int c1 = 0, c2 = 0;
            if (producer) {
                fetch_tile(t0);    // its loads are the oldest: every wait below covers them
                if constexpr (Q_IN_RING) fetch_query_rows();
                if (t0 + 1 < t1) c1 = fetch_tile(t0 + 1);
                if (t0 + 2 < t1) c2 = fetch_tile(t0 + 2);
                await_all_but(c1 + c2);
            }
            __syncthreads();   // the first tile and the query rows are there (every producer's part)
            if (producer) {
                if constexpr (Q_IN_RING) {
                    const uint32_t q_row = (uint32_t)((hg * 16 + n) * ROWB);
                    const uint32_t q_key = (uint32_t)swz_key(n);
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks)
                        st[ks] = *(LDS_AS f32x4*)(qlds + q_row + ((((uint32_t)(4 * ks + g)) ^ q_key) << 4));
                    // (the reads have to be back before the barrier that releases the slot)
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks) asm volatile("" :: "v"(st[ks]));
                }
            }
            __syncthreads();   // the query rows are in registers: their slot joins the ring
            if (producer) {
                // (scores first: with two tiles in flight the new requests would wait for a free
                // place in the memory pipeline and hold the scores back)
                if constexpr (!PROBE) {
                    f32x4 xs;
                    score_block(lds, rb, t0, rows_valid(t0), xs);
                    xbuf[0][hg][rb][lane] = xs;
                    asm volatile("" ::: "memory");
                }
                if (t0 + 3 < t1) c3 = fetch_tile(t0 + 3);
                await_all_but(c2 + c3);   // the second tile is there
            }
        }
        bool jumped = false;
        for (int t = t0; t < t1; ++t) {
            const int par = (t - t0) & 1;
            LDS_AS unsigned char* tile = lds + ((t - t0) % NBUF) * TILE_B;
            const int n_valid = rows_valid(t);
            // tile t's scores are in LDS, tile t + 1 has landed, and everybody is done with tile t - 1
            __syncthreads();
            if (n_valid < TILE_ROWS) {
                // ragged last tile (or a page id outside the pool): rows that are not part of the
                // sequence become zeros so that whatever they hold stays out
                for (int i = tid; i < (TILE_ROWS - n_valid) * CPR; i += ST_THREADS)
                    *(LDS_AS u32x4*)(tile + n_valid * ROWB + i * 16) = (u32x4){0u, 0u, 0u, 0u};
                __syncthreads();
            }
            if (producer) {
                // tile t + 3 into the slot tile t - 1 has left (the first time round it is on its way already)
                const int cn = t == t0 ? c3 : (t + 3 < t1 ? fetch_tile(t + 3) : 0);
                if constexpr (!PROBE) {
                    if (t + 1 < t1) {
                        f32x4 xs;
                        score_block(lds + ((t + 1 - t0) % NBUF) * TILE_B, rb, t + 1, rows_valid(t + 1), xs);
                        xbuf[par ^ 1][hg][rb][lane] = xs;
                    }
                }
                await_all_but(cn);   // tile t + 2 is there before the next barrier
            } else if constexpr (!PROBE) {
                const f32x4 x0 = xbuf[par][hg][0][lane], x1 = xbuf[par][hg][1][lane];
                const float lmax = fmaxf(fmaxf(fmaxf(x0[0], x0[1]), fmaxf(x0[2], x0[3])),
                                         fmaxf(fmaxf(x1[0], x1[1]), fmaxf(x1[2], x1[3])));
                if constexpr (!CAREFUL) {
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
                        for (int i = 0; i < WCT; ++i) st[i] *= alpha;
                        m_run = m_new;
                    }
                }
                accumulate_tile(tile, x0, x1);
            }
        }
        return jumped;
    };

    const bool jumped = sweep(std::false_type{});
    if (jumped) jump_flag = 1;
    __syncthreads();   // every consumer is done with the last tile; nothing is in flight (the producers waited for it)
    if constexpr (PROBE) return;
    if (__builtin_expect(jump_flag != 0, 0)) {
        // ---- careful pass (rare): the same chunk again with a moving reference
        m_run = -INFINITY;
        l_run = 0.f;
#pragma unroll
        for (int i = 0; i < WCT; ++i)
            if (!producer) st[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
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
            const f32x4 o = st[i] * inv;
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

hipError_t launch_decode_stream(const DecodeParams& p, dim3 grid, hipStream_t s)
{
    dim3 block(ST_THREADS);
    if (p.d_c == 512)      decode_stream_kernel<512, false, false><<<grid, block, 0, s>>>(p);
    else if (p.d_c == 256) decode_stream_kernel<256, false, false><<<grid, block, 0, s>>>(p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_decode_stream_balanced(const DecodeParams& p, dim3 grid, hipStream_t s)
{
    dim3 block(ST_THREADS);
    if (!p.plan) return hipErrorInvalidValue;
    if (p.d_c == 512)      decode_stream_kernel<512, false, true><<<grid, block, 0, s>>>(p);
    else if (p.d_c == 256) decode_stream_kernel<256, false, true><<<grid, block, 0, s>>>(p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_decode_stream_probe(const DecodeParams& p, hipStream_t s)
{
    dim3 grid(p.B, p.num_splits), block(ST_THREADS);
    if (p.d_c == 512)      decode_stream_kernel<512, true, false><<<grid, block, 0, s>>>(p);
    else if (p.d_c == 256) decode_stream_kernel<256, true, false><<<grid, block, 0, s>>>(p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace mla
