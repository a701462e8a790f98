// Fused tail of the absorbed attention step: split-KV merge followed by the output
// up-projection (third line of the absorbed equation, Sec. 3.3, inside the brackets; App. A.2.2
// writes the same product as part of W'^O):
//     o_lat[b,h,:] = sum_s e^{lse_s - lse} o_s[b,h,:]          out[b,h,:] = o_lat[b,h,:] . W_UV[h]
// One workgroup = one head x BG batch rows.  The whole W_UV[h] slab ([d_c x 128] bf16, 128 KB at
// d_c = 512) is requested as direct-to-LDS loads right after each wavefront's first partial rows;
// while it is in flight the four wavefronts merge the partial rows (one wavefront per row and block of 256 columns, as in the
// stand-alone merge kernel), write o_lat and leave a bf16 copy in LDS as the A operand.  The
// product then runs on v_mfma_f32_16x16x32_bf16 with the B operand read by transposing LDS
// loads (W is stored k-major).  Compared with the two separate kernels this saves a launch and
// overlaps the two dependent memory latencies.
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

// 16-byte chunk swizzle of slab row r (4 bits): spreads the 16 rows x 32 bytes of one
// transposing read over the banks
__device__ __forceinline__ constexpr int ft_key(int r)
{
    return ((r & 3) << 2) | (((r >> 3) & 1) << 1) | ((r >> 4) & 1);
}

template <int D_C>
__global__ __launch_bounds__(256) void merge_out_proj_kernel(MergeParams p, const uint16_t* W_UV, uint16_t* out, int BG)
{
    constexpr int SLAB_B = D_C * FT_ROWB;             // 131072 / 65536
    constexpr int ARS = D_C * 2 + 16;                 // A tile row stride (padded)
    constexpr int NLOAD = SLAB_B / (256 * 16);        // 32 / 16 direct-to-LDS loads per thread
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

    const int S = p.num_splits;
    constexpr int CB = D_C / 256;
    constexpr int BATCH = 16;
    // wave task = (batch row, block of 256 columns); partial rows [s0, s0 + BATCH) of a task
    auto task_base = [&](int task) {
        const int bl = task / CB, cb = task % CB;
        return part_index(b0 + bl, h, 0, p.H, S) * D_C + cb * 256 + lane * 4;   // element index into the partial rows
    };
    // rows past the last chunk re-read the last one (their weight is zero): no branches, the
    // kernel's code stays short and straight, which matters for a kernel this brief
    auto load_rows = [&](size_t base, int s0, f32x4 (&v)[BATCH]) {
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const float4 r = load_part4<true>(p.o_part, base + (size_t)min(s0 + i, S - 1) * D_C);
            v[i] = (f32x4){r.x, r.y, r.z, r.w};
        }
    };

    // ---- (1) the first task's chunk weights and partial rows are requested ahead of everything
    // else: they come from HBM, the slab mostly from L2 (the workgroups of a head share it).
    // Tasks past the workgroup's batch rows only clear their part of the A tile.
    const int T = nb * CB;                       // tasks with a batch row behind them
    auto request = [&](int task, f32x4 (&v)[BATCH], float& ls) {
        ls = lane < S ? p.lse_part[part_index(b0 + task / CB, h, lane, p.H, S)] : -INFINITY;
        load_rows(task_base(task), 0, v);
    };
    f32x4 va[BATCH], vb[BATCH];
    float lsa = -INFINITY, lsb = -INFINITY;
    if (wave < T) request(wave, va, lsa);
    for (int task = T + wave; task < FT_MAXB * CB; task += 4)
        *(LDS_AS u32x2*)(atile + (task / CB) * ARS + ((task % CB) * 256 + lane * 4) * 2) = (u32x2){0u, 0u};

    // ---- (2) request W_UV[h]: LDS chunk P = row P/16, position P%16 holds chunk (P%16) ^ key(row)
    {
        const unsigned char* src = reinterpret_cast<const unsigned char*>(W_UV + (size_t)h * D_C * FT_N);
        const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
#pragma unroll 4
        for (int k = 0; k < NLOAD; ++k) {
            const int P = (k * 4 + wave) * 64 + lane;
            const int r = P >> 4, pc = P & 15;
            const unsigned char* gp = src + r * FT_ROWB + ((pc ^ ft_key(r)) << 4);
            const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_base + (k * 4 + wave) * 1024);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                         :: "s"(m0v), "v"(gp) : "memory");
        }
    }

    // ---- (3) merge (same arithmetic as the stand-alone merge kernel): this wave's tasks, the
    // next one's rows requested before the current one is reduced
    auto reduce = [&](int task, f32x4 (&v)[BATCH], float ls) {
        const int bl = task / CB, cb = task % CB, b = b0 + bl;
        const size_t base = task_base(task);
        f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
        const ChunkWeights cw = chunk_weights(ls, S);
        for (int s0 = 0; s0 < S; s0 += BATCH) {
            if (s0 > 0) load_rows(base, s0, v);
#pragma unroll
            for (int i = 0; i < BATCH; ++i) {
                // the weight is 0 at and past S; rows of empty chunks were never written,
                // so what was read there is discarded, not multiplied by zero
                const float ws = chunk_weight_at(cw, ls, s0 + i);
                const f32x4 zero = (f32x4){0.f, 0.f, 0.f, 0.f};
                acc += ws * (ws != 0.f ? v[i] : zero);
            }
        }
        const u32x2 packed = (u32x2){f32_to_bf16_bits(acc[0]) | (f32_to_bf16_bits(acc[1]) << 16),
                                    f32_to_bf16_bits(acc[2]) | (f32_to_bf16_bits(acc[3]) << 16)};
        *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(p.o_lat) + ((size_t)b * p.H + h) * D_C + cb * 256 + lane * 4) = packed;
        *(LDS_AS u32x2*)(atile + bl * ARS + (cb * 256 + lane * 4) * 2) = packed;
        if (p.lse && cb == 0 && lane == 0) p.lse[(size_t)b * p.H + h] = cw.z > 0.f ? cw.m + logf(cw.z) : -INFINITY;
    };
    for (int ta = wave; ta < T; ta += 8) {
        const int tb = ta + 4;
        if (tb < T) request(tb, vb, lsb);
        reduce(ta, va, lsa);
        if (tb >= T) break;
        if (tb + 4 < T) request(tb + 4, va, lsa);
        reduce(tb, vb, lsb);
    }

    // ---- (4) slab landed (my loads), then everybody's, and the A tile is complete
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();

    // ---- (5) out = o_lat . W_UV[h]: each wave owns two 16-column tiles
    f32x4 acc[2] = {(f32x4){0.f, 0.f, 0.f, 0.f}, (f32x4){0.f, 0.f, 0.f, 0.f}};
    // transposing read: the lane supplies slab row 32ks + 8g + (n>>2) (+4), 8 bytes at column 4(n&3)
#pragma unroll 4
    for (int ks = 0; ks < D_C / 32; ++ks) {
        const bf16x8 a = *(LDS_AS bf16x8*)(atile + n * ARS + (ks * 32 + g * 8) * 2);
        const int r0 = ks * 32 + g * 8 + (n >> 2);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int cn = (wave * 2 + j) * 2 + ((n & 3) >> 1);      // 16-byte chunk of columns
            const uint32_t sub = (uint32_t)((n & 1) * 8);
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
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int bl = g * 4 + i;
            if (bl < nb)
                out[((size_t)(b0 + bl) * p.H + h) * FT_N + (wave * 2 + j) * 16 + n] = (uint16_t)f32_to_bf16_bits(acc[j][i]);
        }
}

}  // namespace

bool merge_out_proj_supported(const MergeParams& p, int d_head, mla_dtype io)
{
    return !p.plan && io == MLA_BF16 && d_head == FT_N && (p.d_c == 256 || p.d_c == 512) && p.num_splits <= 64 &&
           p.H <= 4096;
}

hipError_t launch_merge_out_proj(const MergeParams& p, const void* W_UV, void* out, hipStream_t s)
{
    // batch rows per workgroup: as few as still gives about one workgroup per CU
    int BG = 1;
    while (BG < FT_MAXB && (long)p.H * ((p.B + BG - 1) / BG) > 256) BG *= 2;
    dim3 grid(p.H, (p.B + BG - 1) / BG), block(256);
    if (p.d_c == 512)
        merge_out_proj_kernel<512><<<grid, block, 0, s>>>(p, static_cast<const uint16_t*>(W_UV), static_cast<uint16_t*>(out), BG);
    else
        merge_out_proj_kernel<256><<<grid, block, 0, s>>>(p, static_cast<const uint16_t*>(W_UV), static_cast<uint16_t*>(out), BG);
    return hipGetLastError();
}

}  // namespace mla
