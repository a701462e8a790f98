// Fused tail of the absorbed attention step: split-KV merge followed by the output
// up-projection (third line of the absorbed equation, Sec. 3.3, inside the brackets; App. A.2.2
// writes the same product as part of W'^O):
//     o_lat[b,h,:] = sum_s e^{lse_s - lse} o_s[b,h,:]          out[b,h,:] = o_lat[b,h,:] . W_UV[h]
// One workgroup = one head x BG batch rows, 16 wavefronts.  The whole W_UV[h] slab ([d_c x 128]
// bf16, 128 KB at d_c = 512) is requested as direct-to-LDS loads right after each wavefront's first
// partial rows; while it is in flight the wavefronts merge the partial rows (one wavefront per row
// and block of 256 columns, as in the stand-alone merge kernel: with 16 wavefronts the 16 tasks of
// 8 rows x 512 or 16 rows x 256 columns wait for memory once, side by side, where four wavefronts
// waited four times in a row), write o_lat and leave a bf16 copy in LDS as the A operand.  The
// product then runs on v_mfma_f32_16x16x32_bf16 (eight wavefronts, one tile of 16 columns each)
// with the B operand read by transposing LDS loads (W is stored k-major).  Compared with the two separate kernels this saves a launch and
// overlaps the two dependent memory latencies.  PLAN = true reads the partials where the balanced
// partition's plan puts them (a sequence's chunks one slot apart, any number of them).
#include "mla_internal.h"

namespace mla {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
#define LDS_AS __attribute__((address_space(3)))

constexpr int FT_N = 128;            // d_head
constexpr int FT_ROWB = FT_N * 2;    // bytes per W row in LDS (unpadded: filled by direct-to-LDS loads)
constexpr int FT_MAXB = 16;          // batch rows per workgroup (one MFMA M tile)
constexpr int FT_WAVES = 16;         // wavefronts per workgroup
constexpr int FT_THREADS = FT_WAVES * 64;

// 16-byte chunk swizzle of slab row r (4 bits): spreads the 16 rows x 32 bytes of one
// transposing read over the banks
__device__ __forceinline__ constexpr int ft_key(int r)
{
    return ((r & 3) << 2) | (((r >> 3) & 1) << 1) | ((r >> 4) & 1);
}

template <int D_C, bool PLAN>
__global__ __launch_bounds__(FT_THREADS) void merge_out_proj_kernel(MergeParams p, const uint16_t* W_UV, uint16_t* out, int BG)
{
    constexpr int SLAB_B = D_C * FT_ROWB;             // 131072 / 65536
    constexpr int ARS = D_C * 2 + 16;                 // A tile row stride (padded)
    constexpr int NLOAD = SLAB_B / (FT_THREADS * 16); // 8 / 4 direct-to-LDS loads per thread
    __shared__ __attribute__((aligned(1024))) unsigned char smem[SLAB_B + FT_MAXB * ARS];
    LDS_AS unsigned char* lds = (LDS_AS unsigned char*)smem;
    LDS_AS unsigned char* atile = lds + SLAB_B;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    // workgroups of one head have linear ids that differ by a multiple of H: they land on the
    // same XCD (ids are dealt round-robin over the 8 XCDs and H is a multiple of 8 for the
    // usual shapes) and share the slab in its L2
    const int h = blockIdx.x;
    const int b0 = blockIdx.y * BG;
    const int nb = min(BG, p.B - b0);

    constexpr int CB = D_C / 256;
    constexpr int BATCH = 16;
    // balanced partition: lane l holds the plan entry of batch row b0 + l (one load for the
    // workgroup's rows, ahead of everything that depends on it)
    int plan_first = 0, plan_count = 0;
    if constexpr (PLAN) {
        if (lane < nb) {
            plan_first = p.plan[2 * (b0 + lane)];
            plan_count = p.plan[2 * (b0 + lane) + 1];
        }
    }
    // the chunks of batch row bl (wave-uniform)
    auto span_of = [&](int bl) -> ChunkSpan {
        if constexpr (PLAN) {
            const int l = __builtin_amdgcn_readfirstlane(bl);
            return planned_span(__builtin_amdgcn_readlane(plan_first, l), __builtin_amdgcn_readlane(plan_count, l), p, h);
        } else {
            return ChunkSpan{part_index(b0 + bl, h, 0, p.H, p.num_splits), 1, p.num_splits};
        }
    };
    // wave task = (batch row, block of 256 columns); partial rows [s0, s0 + BATCH) of a task
    auto task_base = [&](const ChunkSpan& c, int task) {
        return c.first * D_C + (task % CB) * 256 + lane * 4;   // element index into the partial rows
    };
    // rows past the last chunk re-read the last one (their weight is zero): no branches, the
    // kernel's code stays short and straight, which matters for a kernel this brief
    auto load_rows = [&](const ChunkSpan& c, size_t base, int s0, f32x4 (&v)[BATCH]) {
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const float4 r = load_part4<true>(p.o_part, base + (size_t)max(0, min(s0 + i, c.S - 1)) * (c.step * D_C));
            v[i] = (f32x4){r.x, r.y, r.z, r.w};
        }
    };

    // ---- (1) the first task's chunk weights and partial rows are requested ahead of everything
    // else: they come from HBM, the slab mostly from L2 (the workgroups of a head share it).
    // Tasks past the workgroup's batch rows only clear their part of the A tile.
    const int T = nb * CB;                       // tasks with a batch row behind them
    auto request = [&](int task, f32x4 (&v)[BATCH], float& ls) {
        const ChunkSpan c = span_of(task / CB);
        ls = span_lse(p.lse_part, c, 0, lane);
        load_rows(c, task_base(c, task), 0, v);
    };
    f32x4 va[BATCH];
    float lsa = -INFINITY;
    if (wave < T) request(wave, va, lsa);
    for (int task = T + wave; task < FT_MAXB * CB; task += FT_WAVES)
        *(LDS_AS u32x2*)(atile + (task / CB) * ARS + ((task % CB) * 256 + lane * 4) * 2) = (u32x2){0u, 0u};

    // ---- (2) request W_UV[h]: LDS chunk P = row P/16, position P%16 holds chunk (P%16) ^ key(row)
    {
        const unsigned char* src = reinterpret_cast<const unsigned char*>(W_UV + (size_t)h * D_C * FT_N);
        const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
#pragma unroll
        for (int k = 0; k < NLOAD; ++k) {
            const int P = (k * FT_WAVES + wave) * 64 + lane;
            const int r = P >> 4, pc = P & 15;
            const unsigned char* gp = src + r * FT_ROWB + ((pc ^ ft_key(r)) << 4);
            const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_base + (k * FT_WAVES + wave) * 1024);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                         :: "s"(m0v), "v"(gp) : "memory");
        }
    }

    // ---- (3) merge (same arithmetic as the stand-alone merge kernel): this wave's tasks (one, or
    // two for 16 batch rows of 512 columns)
    auto reduce = [&](int task, f32x4 (&v)[BATCH], float ls0) {
        const int bl = task / CB, cb = task % CB, b = b0 + bl;
        const ChunkSpan c = span_of(bl);
        const size_t base = task_base(c, task);
        f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
        const ChunkWeights cw = PLAN ? span_weights(p.lse_part, c, ls0, lane) : chunk_weights(ls0, c.S);
        for (int blk = 0; blk < c.S; blk += 64) {      // one block unless the plan gives a sequence more than 64 chunks
            const float ls = blk ? span_lse(p.lse_part, c, blk, lane) : ls0;
            for (int s0 = 0; s0 < min(64, c.S - blk); s0 += BATCH) {
                if (blk + s0 > 0) load_rows(c, base, blk + s0, v);
#pragma unroll
                for (int i = 0; i < BATCH; ++i) {
                    // the weight is 0 at and past S; rows of empty chunks were never written,
                    // so what was read there is discarded, not multiplied by zero
                    const float ws = chunk_weight_at(cw, ls, s0 + i);
                    const f32x4 zero = (f32x4){0.f, 0.f, 0.f, 0.f};
                    acc += ws * (ws != 0.f ? v[i] : zero);
                }
            }
        }
        const u32x2 packed = (u32x2){f32_to_bf16_bits(acc[0]) | (f32_to_bf16_bits(acc[1]) << 16),
                                    f32_to_bf16_bits(acc[2]) | (f32_to_bf16_bits(acc[3]) << 16)};
        *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(p.o_lat) + ((size_t)b * p.H + h) * D_C + cb * 256 + lane * 4) = packed;
        *(LDS_AS u32x2*)(atile + bl * ARS + (cb * 256 + lane * 4) * 2) = packed;
        if (p.lse && cb == 0 && lane == 0) p.lse[(size_t)b * p.H + h] = cw.z > 0.f ? cw.m + logf(cw.z) : -INFINITY;
    };
    for (int task = wave; task < T; task += FT_WAVES) {
        if (task != wave) request(task, va, lsa);
        reduce(task, va, lsa);
    }

    // ---- (4) slab landed (my loads), then everybody's, and the A tile is complete
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();

    // ---- (5) out = o_lat . W_UV[h]: wavefronts 0..7 own one 16-column tile each, as two
    // interleaved chains over the even and the odd k-steps
    if (wave >= FT_N / 16) return;
    f32x4 acc[2] = {(f32x4){0.f, 0.f, 0.f, 0.f}, (f32x4){0.f, 0.f, 0.f, 0.f}};
    // transposing read: the lane supplies slab row 32ks + 8g + (n>>2) (+4), 8 bytes at column 4(n&3)
    const int cn = wave * 2 + ((n & 3) >> 1);      // 16-byte chunk of columns
    const uint32_t sub = (uint32_t)((n & 1) * 8);
#pragma unroll 4
    for (int ks = 0; ks < D_C / 32; ks += 2) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const bf16x8 a = *(LDS_AS bf16x8*)(atile + n * ARS + ((ks + j) * 32 + g * 8) * 2);
            const int r0 = (ks + j) * 32 + g * 8 + (n >> 2);
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (LDS_AS s16x4*)(lds + r0 * FT_ROWB + ((cn ^ ft_key(r0)) << 4) + sub));
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (LDS_AS s16x4*)(lds + (r0 + 4) * FT_ROWB + ((cn ^ ft_key(r0 + 4)) << 4) + sub));
            s16x8 bb = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, bb), acc[j], 0, 0, 0);
        }
    }
    // D: rows 4g..4g+3 (batch rows of this workgroup) of column n
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int bl = g * 4 + i;
        if (bl < nb)
            out[((size_t)(b0 + bl) * p.H + h) * FT_N + wave * 16 + n] = (uint16_t)f32_to_bf16_bits(acc[0][i] + acc[1][i]);
    }
}

}  // namespace

bool merge_out_proj_supported(const MergeParams& p, int d_head, mla_dtype io)
{
    return io == MLA_BF16 && d_head == FT_N && (p.d_c == 256 || p.d_c == 512) && (p.plan || p.num_splits <= 64) &&
           p.H <= 4096;
}

hipError_t launch_merge_out_proj(const MergeParams& p, const void* W_UV, void* out, hipStream_t s)
{
    // batch rows per workgroup: as few as still gives about one workgroup per CU
    int BG = 1;
    while (BG < FT_MAXB && (long)p.H * ((p.B + BG - 1) / BG) > 256) BG *= 2;
    dim3 grid(p.H, (p.B + BG - 1) / BG), block(FT_THREADS);
    const uint16_t* W = static_cast<const uint16_t*>(W_UV);
    uint16_t* o = static_cast<uint16_t*>(out);
    if (p.d_c == 512 && p.plan)  merge_out_proj_kernel<512, true><<<grid, block, 0, s>>>(p, W, o, BG);
    else if (p.d_c == 512)       merge_out_proj_kernel<512, false><<<grid, block, 0, s>>>(p, W, o, BG);
    else if (p.plan)             merge_out_proj_kernel<256, true><<<grid, block, 0, s>>>(p, W, o, BG);
    else                         merge_out_proj_kernel<256, false><<<grid, block, 0, s>>>(p, W, o, BG);
    return hipGetLastError();
}

}  // namespace mla
