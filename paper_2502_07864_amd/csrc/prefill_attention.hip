// Causal attention of the MHA-paradigm prefill (Sec. 3.3, first of the two attention equations) over
// the keys and values materialised per (sequence, head) by prefill.hip: rows of 320 bf16 values,
// [k = W^{UK}_h c_j ; k^R_j (128 + 64) | v = W^{UV}_h c_j (128)], in pages of 64 rows, one pseudo-
// sequence per (sequence, head).  Query token i of T sees the rows 0 .. L - T + i.
//
//     S^T [keys x queries]  = K [keys x 192] . Q^T [192 x queries]
//     O^T [128 x queries]  += V^T [128 x keys] . P^T [keys x queries]
//
// Workgroup = 128 query rows of one (sequence, head) x all the keys they see; 4 wavefronts, each
// with 32 query rows of its own (two groups of 16) and a private running softmax, so the only
// workgroup barrier per tile is the one that publishes the tile (32 keys, direct-to-LDS loads,
// ring of NBUF tiles).  Per tile a wavefront reads the whole tile from LDS once as the A operand
// of the score contraction (two blocks of 16 keys) and once transposed for the value contraction;
// every read feeds two MFMAs (the two query groups).  As in the decode kernels the transposed
// formulation puts queries on the D columns: a lane owns one query per group, the exponentiated
// scores of key blocks 0 and 1 are, as they stand, the B operand of v_mfma_f32_16x16x32_bf16
// (k slot 8g + j = key 4g + j for j < 4, key 16 + 4g + j - 4 otherwise), and two transposing LDS
// reads give the matching V^T.  No rescaling in the loop: the reference of a query is the maximum of
// its first tile; a later score more than 2^64 above it is recorded and the workgroup then redoes
// its keys with the exact maxima (one sweep that only scores, one that accumulates).
#include "mla_internal.h"
#include "mfma_tile.h"

namespace mla {
namespace {

constexpr int PA_ROW = 320;                 // values per materialised row
constexpr int PA_DK = 192;                  // key part
constexpr int PA_DV = 128;                  // value part
constexpr int PA_ROWS = 128;                // query rows per workgroup

template <int NBUF, int WPE>
__global__ __launch_bounds__(MF_THREADS, WPE) void prefill_attention_kernel(DecodeParams p)
{
    constexpr int ROWB = PA_ROW * 2;            // 640 bytes per row: 32 banks mod 64, as the decode tiles
    constexpr int CPR = ROWB / 16;              // 40 chunks of 16 bytes
    constexpr int PAGE_B = 64 * ROWB;
    constexpr int TILE_B = TILE_ROWS * ROWB;    // 20480
    constexpr int NLOAD = TILE_B / (MF_THREADS * 16);   // 5
    constexpr int NKS = PA_DK / 32;             // 6 k-steps of the score contraction
    constexpr int NCT = PA_DV / 16;             // 8 column tiles of the value contraction
    constexpr int VGR = 2;                      // column tiles per read-ahead group (value)
    static_assert(NBUF >= 2 && NBUF <= 4 && (NBUF + 1) * NLOAD < 64, "ring depth; vmcnt is a 6-bit counter");

    __shared__ __attribute__((aligned(1024))) unsigned char smem[NBUF * TILE_B];
    LDS_AS unsigned char* lds = (LDS_AS unsigned char*)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;

    // Workgroup -> (pseudo-sequence, group of 128 query rows).  The groups of one sequence get
    // linear ids 8 apart (ids are dealt round-robin to the 8 XCDs: they run on one XCD and share the
    // sequence's rows in its L2), the groups with the most keys first.
    const int Z = (p.H + PA_ROWS - 1) / PA_ROWS;
    const int id = blockIdx.x, rr = id >> 3;
    const int zi = Z - 1 - rr % Z;
    const int b = (rr / Z) * 8 + (id & 7);
    if (b >= p.B) return;                       // padding of the last group of 8
    const int hb = zi * PA_ROWS;
    const int HL = min(PA_ROWS, p.H - hb);      // query rows of this workgroup
    // rows of q / out: sequence b stands for (b / q_inner, b % q_inner), its tokens q_inner rows apart
    const size_t io_base = (size_t)(b / p.q_inner) * p.H * p.q_inner + (size_t)(b % p.q_inner);
    auto io_row = [&](int h) -> size_t { return io_base + (size_t)h * p.q_inner; };

    const CONST_AS int32_t* ptab = (const CONST_AS int32_t*)(p.page_table + (size_t)b * p.max_pages);
    const int L = max(0, min(p.seq_lens[b], p.max_pages * 64));

    // ---- this wave's 32 query rows -> registers (B operands of the score contraction)
    bf16x8 qreg[2][NKS];
    {
        const uint16_t* qa = static_cast<const uint16_t*>(p.q_abs);
        const uint16_t* qr = static_cast<const uint16_t*>(p.q_rope);
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) {
            const int row = wave * 32 + hi * 16 + n;
            const size_t qrow = io_row(hb + min(row, HL - 1));
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const uint16_t* src = ks < 4 ? qa + qrow * 128 + ks * 32 + g * 8 : qr + qrow * 64 + (ks - 4) * 32 + g * 8;
                const uint4 v = *reinterpret_cast<const uint4*>(src);
                qreg[hi][ks] = __builtin_bit_cast(bf16x8, row < HL ? v : make_uint4(0u, 0u, 0u, 0u));
            }
        }
    }

    // keys [0, row1): what the last query row of the workgroup sees (the rows are ordered by token)
    const int row1 = min(L, visible_rows(p, L, min(hb + PA_ROWS, p.H) - 1));
    auto store_nothing = [&]() {                // zeros and -inf for the rows of this workgroup
        for (int i = tid; i < HL * (PA_DV / 4); i += MF_THREADS)
            *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(p.o_final) + io_row(hb + i / (PA_DV / 4)) * PA_DV +
                                      (i % (PA_DV / 4)) * 4) = (u32x2){0u, 0u};
        if (tid < HL && p.lse_final) p.lse_final[io_row(hb + tid)] = -INFINITY;
    };
    if (row1 <= 0) {
        store_nothing();
        return;
    }
    const int t1 = (row1 + TILE_ROWS - 1) / TILE_ROWS;            // tiles [0, t1)
    // first key that some query row of this workgroup must not see (its first row sees the least)
    const int causal_from = visible_rows(p, L, hb);

    // ---- tile staging: direct-to-LDS 128-bit loads, chunk swizzle as in the decode kernels
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
    uint32_t goff[NLOAD];
#pragma unroll
    for (int k = 0; k < NLOAD; ++k) {
        const int P = (k * 4 + wave) * 64 + lane;
        const int r = P / CPR, pc = P % CPR;
        goff[k] = (uint32_t)(r * ROWB + ((pc ^ swz_key(r)) << 4));
    }
    const unsigned char* kv = static_cast<const unsigned char*>(p.kv);
    auto rows_valid = [&](int t) {
        const int page = ptab[t >> 1];
        return (page >= 0 && page < p.num_pages) ? min(TILE_ROWS, row1 - t * TILE_ROWS) : 0;
    };
    auto fetch_tile = [&](int t) -> int {       // number of loads this thread issued (0 or NLOAD; uniform)
        if (rows_valid(t) <= 0) return 0;       // a page that was skipped is never dereferenced
        const unsigned char* src = kv + (size_t)ptab[t >> 1] * PAGE_B + (size_t)(t & 1) * TILE_B;
        const uint32_t dst = lds_base + (uint32_t)((t % NBUF) * TILE_B + wave * 1024);
#pragma unroll
        for (int k = 0; k < NLOAD; ++k) {
            const unsigned char* gp = src + goff[k];
            const uint32_t m0v = __builtin_amdgcn_readfirstlane(dst + k * 4096);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                         :: "s"(m0v), "v"(gp) : "memory");
        }
        return NLOAD;
    };
    int ahead[NBUF - 1];        // loads issued for the tiles after the one being consumed, oldest first
    bool ring_full = false;
    auto start_ring = [&]() {
        fetch_tile(0);
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i) ahead[i] = 1 + i < t1 ? fetch_tile(1 + i) : 0;
        ring_full = true;
    };
    auto stage_tile = [&](int t, LDS_AS unsigned char* tile) -> int {
        const int n_valid = rows_valid(t);
        int younger = 0;
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i) younger += ahead[i];
        if (NBUF > 3 && younger >= 3 * NLOAD)      wait_vmcnt<3 * NLOAD>();
        else if (NBUF > 2 && younger >= 2 * NLOAD) wait_vmcnt<2 * NLOAD>();
        else if (younger >= NLOAD)                 wait_vmcnt<NLOAD>();
        else                                       wait_vmcnt<0>();
        // after the barrier everybody's loads of tile t have landed and every wave is done with
        // tile t - 1, whose ring slot now receives tile t + NBUF - 1
        __syncthreads();
        if (!ring_full) {
            const int tn = t + NBUF - 1;
            ahead[NBUF - 2] = tn < t1 ? fetch_tile(tn) : 0;
        }
        ring_full = false;
        if (n_valid < TILE_ROWS) {              // ragged last tile, or a skipped page: zeros, whatever the rows hold
            for (int i = tid; i < (TILE_ROWS - n_valid) * CPR; i += MF_THREADS)
                *(LDS_AS u32x4*)(tile + n_valid * ROWB + i * 16) = (u32x4){0u, 0u, 0u, 0u};
            __syncthreads();
        }
#pragma unroll
        for (int i = 0; i < NBUF - 2; ++i) ahead[i] = ahead[i + 1];
        ahead[NBUF - 2] = 0;
        return n_valid;
    };

    start_ring();
    // pin the completion of the query loads here, outside the tile loop
#pragma unroll
    for (int hi = 0; hi < 2; ++hi)
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) asm volatile("" :: "v"(qreg[hi][ks]));

    // ---- per-lane state: this lane's queries = column n of the D tiles of the two groups
    float m_ref[2] = {-INFINITY, -INFINITY};   // reference of the exponentials (log2 units)
    float l_run[2] = {0.f, 0.f};               // this lane's share of the normaliser (its 8 keys per tile)
    f32x4 oacc[2][NCT];
#pragma unroll
    for (int hi = 0; hi < 2; ++hi)
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) oacc[hi][ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const float sc = p.scale * LOG2E;
    const int my_row = wave * 32 + n;           // + 16 hi; local to the workgroup

    // score A operand: key row 16 rb + n, chunk 4 ks + g
    const uint32_t a_key = (uint32_t)swz_key(n);
    uint32_t a_base[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) a_base[e] = (uint32_t)(n * ROWB) + ((((uint32_t)(4 * e + g)) ^ a_key) << 4);
    // value A operand (transposing reads): the lane supplies key row 4g + (n>>2) (and 16 more),
    // 8 bytes at value column 16 ct + 4 (n&3)
    const uint32_t v_key = (uint32_t)swz_key(g * 4 + (n >> 2));
    uint32_t v_base[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        v_base[e] = (uint32_t)((g * 4 + (n >> 2)) * ROWB) + ((((uint32_t)(2 * e) + (uint32_t)((n & 3) >> 1)) ^ v_key) << 4) +
                    (uint32_t)((n & 1) * 8) + (uint32_t)(PA_DK * 2);

    // S^T for the tile's 32 keys x this wave's 32 queries, log2 units, keys a query must not see
    // (or that are not there) at -inf.  x[rb][hi][i] = key 16 rb + 4g + i, query 16 hi + n.
    auto score_tile = [&](LDS_AS unsigned char* tile, int t, int n_valid, float (&x)[2][2][4]) {
        f32x4 sacc[2][2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int hi = 0; hi < 2; ++hi) sacc[rb][hi] = (f32x4){0.f, 0.f, 0.f, 0.f};
        bf16x8 a0[2][NKS];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
                a0[rb][ks] = *(LDS_AS bf16x8*)(tile + rb * 16 * ROWB + a_base[ks & 1] + (ks >> 1) * 128);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s0 = 0; s0 < NKS; s0 += 2) {
#pragma unroll
            for (int ks = s0 + 2; ks < s0 + 4 && ks < NKS; ++ks)
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
                    a0[rb][ks] = *(LDS_AS bf16x8*)(tile + rb * 16 * ROWB + a_base[ks & 1] + (ks >> 1) * 128);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = s0; ks < s0 + 2 && ks < NKS; ++ks)
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int hi = 0; hi < 2; ++hi)
                        sacc[rb][hi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[rb][ks], qreg[hi][ks], sacc[rb][hi], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int hi = 0; hi < 2; ++hi)
#pragma unroll
                for (int i = 0; i < 4; ++i) x[rb][hi][i] = sacc[rb][hi][i] * sc;
        if (n_valid < TILE_ROWS || (t + 1) * TILE_ROWS > causal_from) {
            // ragged last tile, and the upper limit of each query (the sum runs up to its own position)
#pragma unroll
            for (int hi = 0; hi < 2; ++hi) {
                const int seen = min(n_valid, visible_rows(p, L, hb + my_row + hi * 16) - t * TILE_ROWS);
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (rb * 16 + g * 4 + i >= seen) x[rb][hi][i] = -INFINITY;
            }
        }
    };
    auto lane_max = [&](const float (&x)[2][2][4], int hi) {
        return fmaxf(fmaxf(fmaxf(x[0][hi][0], x[0][hi][1]), fmaxf(x[0][hi][2], x[0][hi][3])),
                     fmaxf(fmaxf(x[1][hi][0], x[1][hi][1]), fmaxf(x[1][hi][2], x[1][hi][3])));
    };
    // maximum over the four lane groups (all 32 keys of the tile), on every lane
    auto over_groups = [&](float v) {
        v = fmaxf(v, __shfl_xor(v, 16));
        return fmaxf(v, __shfl_xor(v, 32));
    };

    // weights against m_ref (rounded to bf16; the normaliser sums exactly the rounded weights), then
    // O^T += V^T . P^T with the transposing reads one group of four column tiles ahead
    auto accumulate_tile = [&](LDS_AS unsigned char* tile, const float (&x)[2][2][4]) {
        bf16x8 pb[2];
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) {
            const float m_use = m_ref[hi] == -INFINITY ? 0.f : m_ref[hi];
            uint32_t w[4];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                w[2 * rb]     = pack_bf16x2(fast_exp2(x[rb][hi][0] - m_use), fast_exp2(x[rb][hi][1] - m_use));
                w[2 * rb + 1] = pack_bf16x2(fast_exp2(x[rb][hi][2] - m_use), fast_exp2(x[rb][hi][3] - m_use));
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) l_run[hi] += bf16_bits_to_f32(w[j] & 0xFFFFu) + bf16_bits_to_f32(w[j] >> 16);
            pb[hi] = __builtin_bit_cast(bf16x8, (u32x4){w[0], w[1], w[2], w[3]});
        }
        s16x4 lo[NCT], up[NCT];
#pragma unroll
        for (int ct = 0; ct < VGR; ++ct) {
            lo[ct] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(tile + v_base[ct & 3] + (ct >> 2) * 128));
            up[ct] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(tile + v_base[ct & 3] + (ct >> 2) * 128 + 16 * ROWB));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c0 = 0; c0 < NCT; c0 += VGR) {
#pragma unroll
            for (int ct = c0 + VGR; ct < c0 + 2 * VGR && ct < NCT; ++ct) {
                lo[ct] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(tile + v_base[ct & 3] + (ct >> 2) * 128));
                up[ct] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(tile + v_base[ct & 3] + (ct >> 2) * 128 + 16 * ROWB));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ct = c0; ct < c0 + VGR && ct < NCT; ++ct) {
                const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo[ct], up[ct], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int hi = 0; hi < 2; ++hi)
                    oacc[hi][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb[hi], oacc[hi][ct], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- one sweep over the keys.  accumulate = false: only the exact maximum of every query is
    // collected (into m_ref, per lane).  Returns whether some score exceeded its reference by more
    // than FAST_GAP.
    auto sweep = [&](bool accumulate) -> bool {
        bool jumped = false;
        for (int t = 0; t < t1; ++t) {
            LDS_AS unsigned char* tile = lds + (t % NBUF) * TILE_B;
            const int n_valid = stage_tile(t, tile);
            float x[2][2][4];
            score_tile(tile, t, n_valid, x);
            const float lm[2] = {lane_max(x, 0), lane_max(x, 1)};
            if (!accumulate) {
                m_ref[0] = fmaxf(m_ref[0], lm[0]);
                m_ref[1] = fmaxf(m_ref[1], lm[1]);
                continue;
            }
            if (__any(m_ref[0] == -INFINITY || m_ref[1] == -INFINITY)) {   // as a rule: the first tile only
#pragma unroll
                for (int hi = 0; hi < 2; ++hi) {
                    const float tm = over_groups(lm[hi]);
                    if (m_ref[hi] == -INFINITY) m_ref[hi] = tm;
                }
            }
            jumped |= lm[0] > m_ref[0] + FAST_GAP || lm[1] > m_ref[1] + FAST_GAP;
            accumulate_tile(tile, x);
        }
        return jumped;
    };

    bool jumped = sweep(true);
    if (__builtin_expect(__syncthreads_or(jumped), 0)) {
        // ---- careful route (rare): exact maxima first, then the same accumulation against them
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) {
            m_ref[hi] = -INFINITY;
            l_run[hi] = 0.f;
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) oacc[hi][ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
        start_ring();
        sweep(false);
        m_ref[0] = over_groups(m_ref[0]);
        m_ref[1] = over_groups(m_ref[1]);
        __syncthreads();         // every wave is done with the tiles of that sweep
        start_ring();
        sweep(true);
    }
    __syncthreads();             // every wave is done with the tiles: the ring becomes exchange space

    // ---- normalise, round to bf16, transpose through LDS (a lane holds 4 consecutive columns of its
    // query per column tile) and store whole 256-byte rows
    constexpr int RSO = PA_DV * 2 + 16;         // row stride of the transposed block (padded)
    static_assert(4 * 32 * RSO <= NBUF * TILE_B, "exchange space must fit in the tile ring");
    LDS_AS unsigned char* mine = lds + wave * (32 * RSO);
    float lt[2];
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
        float l = l_run[hi] + __shfl_xor(l_run[hi], 16);
        lt[hi] = l + __shfl_xor(l, 32);
        const float inv = lt[hi] > 0.f ? 1.f / lt[hi] : 0.f;
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            const f32x4 v = oacc[hi][ct] * inv;
            *(LDS_AS u32x2*)(mine + (hi * 16 + n) * RSO + (ct * 16 + g * 4) * 2) =
                (u32x2){pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
        }
    }
    const int nrow = min(32, HL - wave * 32);
#pragma unroll
    for (int r0 = 0; r0 < 32; r0 += 4) {
        const int r = r0 + (lane >> 4), c = lane & 15;   // 16 lanes x 16 bytes = one row
        if (r < nrow) {
            const u32x4 v = *(LDS_AS u32x4*)(mine + r * RSO + c * 16);
            *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(p.o_final) + io_row(hb + wave * 32 + r) * PA_DV + c * 8) = v;
        }
    }
    if (g == 0 && p.lse_final) {
#pragma unroll
        for (int hi = 0; hi < 2; ++hi)
            if (my_row + hi * 16 < HL)
                p.lse_final[io_row(hb + my_row + hi * 16)] =
                    lt[hi] > 0.f ? (m_ref[hi] + __builtin_amdgcn_logf(lt[hi])) * LN2 : -INFINITY;
    }
}

}  // namespace

// Causal attention over materialised keys and values: p.B pseudo-sequences ((sequence, head) pairs)
// of p.H query rows each, results straight to o_final / lse_final.
hipError_t launch_prefill_attention(const DecodeParams& p, hipStream_t s)
{
    if (!p.o_final || p.heads != 1 || p.q_inner < 1) return hipErrorInvalidValue;
    const long long Z = (p.H + PA_ROWS - 1) / PA_ROWS;
    const long long nwg = ((long long)p.B + 7) / 8 * 8 * Z;
    if (nwg > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    prefill_attention_kernel<3, 2><<<dim3((unsigned)nwg), dim3(MF_THREADS), 0, s>>>(p);
    return hipGetLastError();
}

}  // namespace mla
