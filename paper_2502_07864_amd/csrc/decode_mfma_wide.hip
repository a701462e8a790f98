// Matrix-core paged decode with 64 query rows per workgroup (bf16 cache, gfx950 / CDNA4): several
// query tokens per sequence (multi-token prediction / speculative decoding) or more than 32 heads.
//
// Same contractions as the 32-row kernel (second line of the absorbed attention equation, Sec. 3.3,
// with one upper limit of the sum per query token):
//     S^T [tok x rows]  = K [tok x (d_c+64)] . Q^T [(d_c+64) x rows]
//     O^T [d_c x rows] += V^T [d_c x tok] . P^T [tok x rows]
// but twice the query rows share every byte that comes from HBM *and* every byte read from LDS:
// the cached rows are still streamed once, and the LDS traffic per tile is that of the 32-row
// kernel, because the work is cut so that no wavefront reads more of a tile than it does there.
//
// Work decomposition (4 wavefronts; wave = (a, hp), hp = pair of 16-row groups of query rows):
//   score phase:  wave (a, hp) scores the 16 tile rows [16a, 16a+16) against the 32 query rows of
//                 pair hp (one A read from LDS feeds two MFMAs), exponentiates against a reference
//                 that both halves share, and leaves the bf16 weights P in a small LDS buffer.
//   value phase:  wave (a, hp) accumulates the d_c/2 columns [a d_c/2, (a+1) d_c/2) for the 32
//                 query rows of pair hp over all 32 tile rows (K = 32: v_mfma_f32_16x16x32_bf16,
//                 one pair of transposing LDS reads feeds two MFMAs).
// Every accumulator is touched by MFMA only; nothing is rescaled in the loop.  The reference of a
// query row is the maximum of its first tile with a visible row (both halves of the tile, exchanged
// through LDS once); a later score that exceeds it by more than FAST_GAP is recorded, and the chunk
// is then redone with the exact maximum of the chunk as the reference (one sweep that only scores,
// one that accumulates).
//
// The k index of the second contraction is laid out so that both operands come out of the first
// one without shuffling: slot 8g + j of lane group g is tile row 4g + j (j < 4) or 16 + 4g + j - 4:
// the first four are what wave a = 0 holds after scoring (D rows 4g..4g+3), the last four what
// wave a = 1 holds, and two transposing reads (rows 4g.., rows 16+4g..) give the matching V^T.
#include "mla_internal.h"
#include "mfma_tile.h"

namespace mla {
namespace {

constexpr int WD_ROWS = 64;      // query rows per workgroup
constexpr int WD_NBUF = 4;       // tiles in the LDS ring

template <int D_C>
__global__ __launch_bounds__(MF_THREADS, 1) void decode_mfma_wide_kernel(DecodeParams p)
{
    constexpr int NBUF = WD_NBUF;
    constexpr int ROW = D_C + 64;               // elements per cache row
    constexpr int ROWB = ROW * 2;               // bytes per row
    constexpr int CPR = ROWB / 16;              // 16-byte chunks per row (72 / 40)
    constexpr int PAGE_B = 64 * ROWB;           // bytes per page
    constexpr int TILE_B = TILE_ROWS * ROWB;    // bytes per tile
    constexpr int NLOAD = TILE_B / (MF_THREADS * 16);  // 16-byte loads per thread per tile (9 / 5)
    constexpr int NKS = ROW / 32;               // k-steps of the score contraction (18 / 10)
    constexpr int CTW = D_C / 32;               // column tiles of the value contraction per wavefront (16 / 8)
    constexpr int SG = NKS % 3 == 0 ? 3 : 2;    // k-steps per read-ahead group (score)
    constexpr int VG = 4;                       // column tiles per read-ahead group (value)
    constexpr int AH = 2;                       // groups the LDS reads run ahead of the MFMAs
    static_assert(2 * NLOAD * 2 < 64, "vmcnt is a 6-bit counter");

    __shared__ __attribute__((aligned(1024))) unsigned char smem[NBUF * TILE_B];
    __shared__ __attribute__((aligned(16))) unsigned char p_smem[2][WD_ROWS * 64];   // weights of two tiles
    __shared__ float xch_smem[2][WD_ROWS];                                           // per-row scalars of the two halves
    LDS_AS unsigned char* lds = (LDS_AS unsigned char*)smem;
    LDS_AS unsigned char* p_lds = (LDS_AS unsigned char*)p_smem;
    LDS_AS float* xch = (LDS_AS float*)xch_smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int a = wave & 1, hp = wave >> 1;
    const int n = lane & 15, g = lane >> 4;

    // Workgroup -> (sequence, chunk, group of 64 query rows).  One group: the two-dimensional grid
    // of the 32-row kernel (sequence rotated by the chunk index).  More: one-dimensional, the
    // groups of a chunk 8 ids apart (same XCD, same time: all but the first find the rows in L2).
    const int Z = (p.H + WD_ROWS - 1) / WD_ROWS;
    int cx = blockIdx.x, cy = blockIdx.y, zi = 0;
    if (Z > 1) {
        const int id = blockIdx.x, r = id >> 3;
        zi = r % Z;
        const int c = (r / Z) * 8 + (id & 7);
        if (c >= p.B * p.num_splits) return;   // padding of the last group of 8
        cx = c % p.B;
        cy = c / p.B;
    }
    const int b = (cx + cy) % p.B, split = cy;
    const int hb = zi * WD_ROWS;
    const int HL = min(WD_ROWS, p.H - hb);     // query rows of this workgroup

    auto o_row = [&](int h) -> uint16_t* {    // partial rows are bf16 (the io dtype of this kernel)
        return static_cast<uint16_t*>(p.o_part) + part_index(b, h, split, p.H, p.num_splits) * D_C;
    };
    auto lse_at = [&](int h) -> float* { return p.lse_part + part_index(b, h, split, p.H, p.num_splits); };

    // read-only tables through the scalar cache (no vector-memory counter involved)
    const CONST_AS int32_t* seq_lens_c = (const CONST_AS int32_t*)p.seq_lens;
    const CONST_AS int32_t* ptab = (const CONST_AS int32_t*)(p.page_table + (size_t)b * p.max_pages);
    const int warm = ptab[min(split * p.chunk_pages, p.max_pages - 1)];
    int L = seq_lens_c[b];

    // ---- the 64 query rows [q_abs | q_rope], laid out like two cache tiles (one row per query
    // row, same chunk swizzle, absent rows zero), travel through the last two ring slots
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    LDS_AS unsigned char* qslot = lds + (NBUF - 2) * TILE_B;
    {
        const unsigned char* qa = static_cast<const unsigned char*>(p.q_abs) + ((size_t)b * p.H + hb) * D_C * 2;
        const unsigned char* qr = static_cast<const unsigned char*>(p.q_rope) + ((size_t)b * p.H + hb) * 128;
        const uint32_t dst = lds_base + (uint32_t)((NBUF - 2) * TILE_B + wave * 1024);
#pragma unroll
        for (int k = 0; k < 2 * NLOAD; ++k) {
            const int P = (k * 4 + wave) * 64 + lane;
            const int r = P / CPR, c = (P % CPR) ^ swz_key(r);
            if (r < HL) {
                const unsigned char* gp = c < D_C / 8 ? qa + ((size_t)r * D_C + c * 8) * 2
                                                      : qr + ((size_t)r * 64 + (c - D_C / 8) * 8) * 2;
                const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst + k * 4096);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                             :: "s"(m0v), "v"(gp) : "memory");
            } else {
                *(LDS_AS u32x4*)(qslot + P * 16) = (u32x4){0u, 0u, 0u, 0u};
            }
        }
    }

    asm volatile("" :: "s"(warm));
    L = max(0, min(L, p.max_pages * 64));
    const int row0 = split * p.chunk_pages * 64;              // first cached row of this chunk
    // one past its last row that some query row of this workgroup sees (the query rows are ordered
    // by token, so the last one sees the most)
    const int row1 = min(min(row0 + p.chunk_pages * 64, L), visible_rows(p, L, min(hb + WD_ROWS, p.H) - 1));
    if (row0 >= row1) {  // nothing to see: weight zero in the merge, partial output never read
        if (tid < HL) *lse_at(hb + tid) = -INFINITY;
        wait_vmcnt<0>();  // the workgroup's LDS must not be released with loads into it in flight
        return;
    }
    const int t0 = row0 / TILE_ROWS;                          // tiles [t0, t1) of the sequence
    const int t1 = (row1 + TILE_ROWS - 1) / TILE_ROWS;
    // first cached row that some query row of this workgroup must not see (its first row sees the least)
    const int causal_from = visible_rows(p, L, hb);

    // ---- tile staging: HBM -> LDS with direct-to-LDS 128-bit loads (as in the 32-row kernel)
    uint32_t goff[NLOAD];
#pragma unroll
    for (int k = 0; k < NLOAD; ++k) {
        int P = (k * 4 + wave) * 64 + lane;
        int r = P / CPR, pc = P % CPR;
        goff[k] = (uint32_t)(r * ROWB + ((pc ^ swz_key(r)) << 4));
    }
    const unsigned char* kv = static_cast<const unsigned char*>(p.kv);
    auto rows_valid = [&](int t) {
        int page = ptab[t >> 1];
        return (page >= 0 && page < p.num_pages) ? min(TILE_ROWS, row1 - t * TILE_ROWS) : 0;
    };
    auto fetch_tile = [&](int t) -> int {
        if (rows_valid(t) <= 0) return 0;   // a page outside the pool is never dereferenced
        const unsigned char* src = kv + (size_t)ptab[t >> 1] * PAGE_B + (size_t)(t & 1) * TILE_B;
        const uint32_t dst = lds_base + (uint32_t)(((t - t0) % NBUF) * TILE_B + wave * 1024);
#pragma unroll
        for (int k = 0; k < NLOAD; ++k) {
            const unsigned char* gp = src + goff[k];
            const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst + k * 4096);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                         :: "s"(m0v), "v"(gp) : "memory");
        }
        return NLOAD;
    };

    // `ahead` holds the loads issued for the tiles after the one being consumed, oldest first
    int ahead[NBUF - 1];
    bool ring_full = false;   // the tile NBUF - 1 ahead has been requested before the first stage step
    // request the first tiles; `upto` of them (the last two slots hold the query rows at first)
    auto start_ring = [&](int upto) -> int {
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i) ahead[i] = 0;
        const int first = fetch_tile(t0);
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i)
            if (1 + i < upto && t0 + 1 + i < t1) ahead[i] = fetch_tile(t0 + 1 + i);
        ring_full = upto == NBUF;
        return first;
    };
    auto wait_younger = [&](int younger) {
        if (younger >= 3 * NLOAD)      wait_vmcnt<3 * NLOAD>();
        else if (younger >= 2 * NLOAD) wait_vmcnt<2 * NLOAD>();
        else if (younger >= NLOAD)     wait_vmcnt<NLOAD>();
        else                           wait_vmcnt<0>();
    };
    // publish tile t (and keep the stream going); returns its number of valid rows
    auto stage_tile = [&](int t, LDS_AS unsigned char* tile) -> int {
        const int n_valid = rows_valid(t);
        int younger = 0;
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i) younger += ahead[i];
        wait_younger(younger);
        // after the barrier everybody's loads of tile t have landed and every wave is done with
        // tile t - 1 (both phases), whose ring slot now receives tile t + NBUF - 1
        __syncthreads();
        if (!ring_full) {
            const int tn = t + NBUF - 1;
            ahead[NBUF - 2] = tn < t1 ? fetch_tile(tn) : 0;
        }
        ring_full = false;
        if (n_valid < TILE_ROWS) {
            for (int i = tid; i < (TILE_ROWS - n_valid) * CPR; i += MF_THREADS)
                *(LDS_AS u32x4*)(tile + n_valid * ROWB + i * 16) = (u32x4){0u, 0u, 0u, 0u};
            __syncthreads();
        }
#pragma unroll
        for (int i = 0; i < NBUF - 2; ++i) ahead[i] = ahead[i + 1];
        ahead[NBUF - 2] = 0;
        return n_valid;
    };

    // ---- query rows -> registers (B operands of the score contraction, resident for the chunk)
    const int first_issued = start_ring(NBUF - 2);
    {
        int later = first_issued;
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i) later += ahead[i];
        wait_younger(later);     // the query rows only: the tile loads requested after them stay in flight
    }
    __syncthreads();
    bf16x8 qreg[2][NKS];
    {
        const uint32_t q_key = (uint32_t)swz_key(n);
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) {
            const uint32_t q_row = (uint32_t)((hp * 32 + hi * 16 + n) * ROWB);
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                qreg[hi][ks] = *(LDS_AS bf16x8*)(qslot + q_row + ((((uint32_t)(4 * ks + g)) ^ q_key) << 4));
        }
    }
    __syncthreads();
    // the two slots join the ring
#pragma unroll
    for (int i = NBUF - 3; i < NBUF - 1; ++i) ahead[i] = t0 + 1 + i < t1 ? fetch_tile(t0 + 1 + i) : 0;
    ring_full = true;

    // ---- per-lane state.  Score phase: this lane's query rows = column n of the two D tiles.
    const int head0 = hp * 32 + n;                    // + 16 hi; local to the workgroup
    float m_ref[2] = {-INFINITY, -INFINITY};          // reference of the exponentials (log2 units), shared by both halves
    float l_run[2] = {0.f, 0.f};                      // this lane's share of the normaliser (its 4 tile rows)
    f32x4 oacc[2][CTW];                               // value phase: columns 16ct + 4g.. of query row n, per 16-row group
#pragma unroll
    for (int hi = 0; hi < 2; ++hi)
#pragma unroll
        for (int ct = 0; ct < CTW; ++ct) oacc[hi][ct] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const float sc = p.scale * LOG2E;
    // score A operand: tile row 16a + n, chunk 4ks + g
    const uint32_t a_row = (uint32_t)((a * 16 + n) * ROWB);
    const uint32_t a_key = (uint32_t)swz_key(n);
    uint32_t a_base[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) a_base[e] = a_row + ((((uint32_t)(4 * e + g)) ^ a_key) << 4);
    // value A operand (transposing reads): the lane supplies tile row 4g + (n>>2) (and 16 more),
    // 8 bytes at element column a d_c/2 + 16ct + 4(n&3)
    const uint32_t v_row = (uint32_t)((g * 4 + (n >> 2)) * ROWB);
    const uint32_t v_key = (uint32_t)swz_key(g * 4 + (n >> 2));
    uint32_t v_base[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        v_base[e] = v_row + ((((uint32_t)(2 * e) + (uint32_t)((n & 3) >> 1)) ^ v_key) << 4) + (uint32_t)((n & 1) * 8) +
                    (uint32_t)(a * D_C);     // column half a starts d_c/2 elements = d_c bytes into the row

    // S^T for this wave's 16 tile rows x 32 query rows, log2 units, rows a query row must not see
    // (or that are not there) at -inf; lmax = maximum over this lane's 4 tile rows per query row
    // (the cross-lane step to the maximum over the wave's 16 rows costs two LDS round trips and is
    // taken only where that maximum is needed)
    auto score_tile = [&](LDS_AS unsigned char* tile, int t, int n_valid, float (&x)[2][4], float (&lmax)[2]) {
        f32x4 sacc[2] = {(f32x4){0.f, 0.f, 0.f, 0.f}, (f32x4){0.f, 0.f, 0.f, 0.f}};
        bf16x8 a0[NKS];
#pragma unroll
        for (int ks = 0; ks < AH * SG && ks < NKS; ++ks)
            a0[ks] = *(LDS_AS bf16x8*)(tile + a_base[ks & 1] + (ks >> 1) * 128);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s0 = 0; s0 < NKS; s0 += SG) {
#pragma unroll
            for (int ks = s0 + AH * SG; ks < s0 + (AH + 1) * SG && ks < NKS; ++ks)
                a0[ks] = *(LDS_AS bf16x8*)(tile + a_base[ks & 1] + (ks >> 1) * 128);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = s0; ks < s0 + SG && ks < NKS; ++ks) {
                sacc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[ks], qreg[0][ks], sacc[0], 0, 0, 0);
                sacc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[ks], qreg[1][ks], sacc[1], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int hi = 0; hi < 2; ++hi)
#pragma unroll
            for (int i = 0; i < 4; ++i) x[hi][i] = sacc[hi][i] * sc;
        if (n_valid < TILE_ROWS || (t + 1) * TILE_ROWS > causal_from) {
            // ragged last tile, and the upper limit of each query row (Eq. "mqa": the sum runs
            // up to the query token's own position)
#pragma unroll
            for (int hi = 0; hi < 2; ++hi) {
                const int seen = min(n_valid, visible_rows(p, L, hb + head0 + hi * 16) - t * TILE_ROWS);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (a * 16 + g * 4 + i >= seen) x[hi][i] = -INFINITY;
            }
        }
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) lmax[hi] = fmaxf(fmaxf(x[hi][0], x[hi][1]), fmaxf(x[hi][2], x[hi][3]));
    };
    // maximum over the four lane groups (the wave's 16 tile rows), on every lane
    auto over_groups = [&](float (&v)[2]) {
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) {
            v[hi] = fmaxf(v[hi], __shfl_xor(v[hi], 16));
            v[hi] = fmaxf(v[hi], __shfl_xor(v[hi], 32));
        }
    };

    // this wave's per-row values v (one per 16-row group; lanes g = 0 write) -> maximum with the
    // other half's, on every lane; one barrier.  The caller guarantees a barrier between two uses.
    auto exchange_max = [&](float (&v)[2]) {
        if (g == 0) {
            xch[a * WD_ROWS + head0] = v[0];
            xch[a * WD_ROWS + head0 + 16] = v[1];
        }
        __syncthreads();
        v[0] = fmaxf(v[0], xch[(a ^ 1) * WD_ROWS + head0]);
        v[1] = fmaxf(v[1], xch[(a ^ 1) * WD_ROWS + head0 + 16]);
    };

    // O^T += V^T . P^T for this wave's column half and its 32 query rows, all 32 tile rows
    auto accumulate_tile = [&](LDS_AS unsigned char* tile, LDS_AS unsigned char* pbuf) {
        const bf16x8 pb0 = *(LDS_AS bf16x8*)(pbuf + (head0) * 64 + g * 16);
        const bf16x8 pb1 = *(LDS_AS bf16x8*)(pbuf + (head0 + 16) * 64 + g * 16);
        s16x4 lo[CTW], hi[CTW];
#pragma unroll
        for (int ct = 0; ct < AH * VG && ct < CTW; ++ct) {
            lo[ct] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(tile + v_base[ct & 3] + (ct >> 2) * 128));
            hi[ct] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(tile + v_base[ct & 3] + (ct >> 2) * 128 + 16 * ROWB));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c0 = 0; c0 < CTW; c0 += VG) {
#pragma unroll
            for (int ct = c0 + AH * VG; ct < c0 + (AH + 1) * VG && ct < CTW; ++ct) {
                lo[ct] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(tile + v_base[ct & 3] + (ct >> 2) * 128));
                hi[ct] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(tile + v_base[ct & 3] + (ct >> 2) * 128 + 16 * ROWB));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ct = c0; ct < c0 + VG && ct < CTW; ++ct) {
                const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo[ct], hi[ct], 0, 1, 2, 3, 4, 5, 6, 7));
                oacc[0][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb0, oacc[0][ct], 0, 0, 0);
                oacc[1][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb1, oacc[1][ct], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- one sweep over the chunk's tiles.  accumulate = false: only the exact maximum of every
    // query row is collected (into m_ref, this wave's rows).  accumulate = true: weights against
    // m_ref and the value contraction; while `need_ref`, m_ref is still being established from
    // the first tile with a visible row.  Returns whether some score exceeded its reference by
    // more than FAST_GAP (this wave's rows).
    auto sweep = [&](bool accumulate, bool need_ref) -> bool {
        bool jumped = false;
        bool row_has_ref = false;          // lane l: query row l has its reference (while need_ref)
        for (int t = t0; t < t1; ++t) {
            LDS_AS unsigned char* tile = lds + ((t - t0) % NBUF) * TILE_B;
            LDS_AS unsigned char* pbuf = p_lds + ((t - t0) & 1) * (WD_ROWS * 64);
            const int n_valid = stage_tile(t, tile);
            float x[2][4], lmax[2];
            score_tile(tile, t, n_valid, x, lmax);
            if (!accumulate) {
                m_ref[0] = fmaxf(m_ref[0], lmax[0]);      // per lane; combined after the sweep
                m_ref[1] = fmaxf(m_ref[1], lmax[1]);
                continue;
            }
            if (need_ref) {
                float both[2] = {lmax[0], lmax[1]};
                over_groups(both);
                exchange_max(both);
                if (m_ref[0] == -INFINITY) m_ref[0] = both[0];
                if (m_ref[1] == -INFINITY) m_ref[1] = both[1];
                // every wave looks at all 64 rows, so all of them drop the exchange at the same tile
                row_has_ref |= fmaxf(xch[lane], xch[WD_ROWS + lane]) != -INFINITY;
                need_ref = __ballot(row_has_ref) != ~0ull;
            }
#pragma unroll
            for (int hi = 0; hi < 2; ++hi) {
                jumped |= lmax[hi] > m_ref[hi] + FAST_GAP;
                const float m_use = m_ref[hi] == -INFINITY ? 0.f : m_ref[hi];
                const uint32_t p01 = pack_bf16x2(fast_exp2(x[hi][0] - m_use), fast_exp2(x[hi][1] - m_use));
                const uint32_t p23 = pack_bf16x2(fast_exp2(x[hi][2] - m_use), fast_exp2(x[hi][3] - m_use));
                // the normaliser sums exactly the rounded weights that get multiplied
                l_run[hi] += (bf16_bits_to_f32(p01 & 0xFFFFu) + bf16_bits_to_f32(p01 >> 16)) +
                             (bf16_bits_to_f32(p23 & 0xFFFFu) + bf16_bits_to_f32(p23 >> 16));
                // k slots 4a .. 4a+3 of lane group g of query row head0 + 16 hi
                *(LDS_AS u32x2*)(pbuf + (head0 + hi * 16) * 64 + g * 16 + a * 8) = (u32x2){p01, p23};
            }
            __syncthreads();     // both halves' weights of this tile are in place
            accumulate_tile(tile, pbuf);
        }
        return jumped;
    };

    bool jumped = sweep(true, true);
    if (__builtin_expect(__syncthreads_or(jumped), 0)) {
        // ---- careful route (rare): exact maxima first, then the same accumulation against them
        m_ref[0] = m_ref[1] = -INFINITY;
        l_run[0] = l_run[1] = 0.f;
#pragma unroll
        for (int hi = 0; hi < 2; ++hi)
#pragma unroll
            for (int ct = 0; ct < CTW; ++ct) oacc[hi][ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
        start_ring(NBUF);
        sweep(false, false);
        __syncthreads();         // every wave is done with the tiles, and with the exchange area
        over_groups(m_ref);
        exchange_max(m_ref);
        start_ring(NBUF);
        sweep(true, false);
    }
    __syncthreads();             // every wave is done with the tiles: the ring becomes exchange space

    // ---- normalise and write the partial: this wave holds columns [a d_c/2, +d_c/2) of its 32
    // query rows, complete.  The normaliser is the sum of both halves' shares.
    float l_w[2];
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
        float l = l_run[hi] + __shfl_xor(l_run[hi], 16);
        l_w[hi] = l + __shfl_xor(l, 32);
    }
    if (g == 0) {
        xch[a * WD_ROWS + head0] = l_w[0];
        xch[a * WD_ROWS + head0 + 16] = l_w[1];
    }
    __syncthreads();
    float inv[2], lt[2];
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
        lt[hi] = l_w[hi] + xch[(a ^ 1) * WD_ROWS + head0 + hi * 16];
        inv[hi] = lt[hi] > 0.f ? 1.f / lt[hi] : 0.f;
    }
    // transpose through LDS (a lane holds 4 consecutive columns of query row n per column tile,
    // which written straight out would give 8-byte pieces), rounded to bf16, and store whole runs
    constexpr int CW = D_C / 2;                 // columns per wavefront
    constexpr int RSO = CW * 2 + 32;            // row stride of the transposed block in bytes (padded)
    static_assert(4 * 32 * RSO <= NBUF * TILE_B, "exchange space must fit in the tile ring");
    LDS_AS unsigned char* mine = lds + wave * (32 * RSO);
#pragma unroll
    for (int hi = 0; hi < 2; ++hi)
#pragma unroll
        for (int ct = 0; ct < CTW; ++ct)
        {
            const f32x4 o = oacc[hi][ct] * inv[hi];
            *(LDS_AS u32x2*)(mine + (hi * 16 + n) * RSO + (ct * 16 + g * 4) * 2) =
                (u32x2){pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
        }
    constexpr int LPR = CW / 8;                 // lanes (of 16 bytes = 8 bf16) covering one row of the half (32 / 16)
    constexpr int RPI = 64 / LPR;               // rows one store instruction covers (2 or 4)
    const int nrow = min(32, HL - hp * 32);
    // reads in batches of eight, then their stores, from one base address and a row stride
    {
        const size_t row_stride = (size_t)p.num_splits * D_C;   // elements between the partial rows of consecutive query rows
        const int rl = lane / LPR, c = lane % LPR;
        uint16_t* dst0 = o_row(hb + hp * 32) + (size_t)rl * row_stride + a * CW + c * 8;
        constexpr int NI = 32 / RPI;               // store instructions (16 / 8)
#pragma unroll
        for (int j0 = 0; j0 < NI; j0 += 8) {
            u32x4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = *(LDS_AS u32x4*)(mine + ((j0 + j) * RPI + rl) * RSO + c * 16);
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if ((j0 + j) * RPI + rl < nrow)
                    __builtin_nontemporal_store(v[j], reinterpret_cast<u32x4*>(dst0 + (size_t)((j0 + j) * RPI) * row_stride));
        }
    }
    if (a == 0 && g == 0) {
#pragma unroll
        for (int hi = 0; hi < 2; ++hi)
            if (head0 + hi * 16 < HL)
                *lse_at(hb + head0 + hi * 16) = lt[hi] > 0.f ? (m_ref[hi] + __builtin_amdgcn_logf(lt[hi])) * LN2 : -INFINITY;
    }
}

}  // namespace

bool decode_mfma_wide_supported(const DecodeParams& p, mla_dtype io, mla_dtype cache)
{
    return io == MLA_BF16 && cache == MLA_BF16 && p.page_size == 64 && p.d_rope == 64 &&
           (p.d_c == 256 || p.d_c == 512) && p.H > 32 &&
           ((long long)p.B * p.num_splits + 7) / 8 * 8 * ((p.H + WD_ROWS - 1) / WD_ROWS) <= 0x7FFFFFFFLL;
}

hipError_t launch_decode_mfma_wide(const DecodeParams& p, hipStream_t s)
{
    const long long nchunk = (long long)p.B * p.num_splits, Z = (p.H + WD_ROWS - 1) / WD_ROWS;
    dim3 grid(p.B, p.num_splits), block(MF_THREADS);
    if (Z > 1) grid = dim3((unsigned)((nchunk + 7) / 8 * 8 * Z));
    if (p.d_c == 512)      decode_mfma_wide_kernel<512><<<grid, block, 0, s>>>(p);
    else if (p.d_c == 256) decode_mfma_wide_kernel<256><<<grid, block, 0, s>>>(p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace mla
