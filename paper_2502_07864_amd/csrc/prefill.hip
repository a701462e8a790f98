// Prefill in the "MHA paradigm" (Sec. 3.3, first of the two attention equations): keys and values
// are materialised per head from the cached latent rows,
//     k_{j,h} = [W^{UK}_h c_j ; k^R_j],        v_{j,h} = W^{UV}_h c_j,
// and the prompt's tokens attend causally to them.  This file holds the two kernels that build
// the materialised rows; the attention itself runs on the 64-row matrix-core kernel, for which one
// (sequence, head) pair is a sequence of its own whose cached rows are [k (128 + 64) | v (128)].
//
//   prefill_weights_kernel      Wcat[h] = [W^{UK}_h ; W^{UV}_h] as 256 rows of d_c values each (the
//                               value projection is stored k-major by the caller and is transposed
//                               here once), so that both products read their weights row-wise.
//   prefill_materialise_kernel  one workgroup per (page, sequence, head):
//                               Y^T [256 x 64 tokens] = Wcat[h] [256 x d_c] . C^T [d_c x 64 tokens]
//                               on v_mfma_f32_16x16x32_bf16; a wavefront owns 16 tokens, keeps
//                               their latent rows in registers as the B operand and walks the 16
//                               row tiles of Wcat[h]; rows are rounded to bf16 and stored as
//                               [k_nope | k_rope (copied from the cache) | v].
#include "mla_internal.h"
#include "mfma_tile.h"

namespace mla {
namespace {

constexpr int PF_ROW = 320;     // values per materialised row: 128 + 64 | 128
constexpr int PF_DH = 128;      // head dimension

__global__ __launch_bounds__(256) void prefill_weights_kernel(const uint16_t* W_UK, const uint16_t* W_UV,
                                                              uint16_t* Wcat, int d_c)
{
    // grid (256 rows, heads); threads over the d_c columns of one row
    const int r = blockIdx.x, h = blockIdx.y;
    uint16_t* dst = Wcat + ((size_t)h * 256 + r) * d_c;
    for (int c = threadIdx.x; c < d_c; c += blockDim.x)
        dst[c] = r < PF_DH ? W_UK[((size_t)h * PF_DH + r) * d_c + c]                  // W_UK[h] is [d_head x d_c]
                           : W_UV[((size_t)h * d_c + c) * PF_DH + (r - PF_DH)];       // W_UV[h] is [d_c x d_head]
}

template <int D_C>
__global__ __launch_bounds__(256) void prefill_materialise_kernel(const uint16_t* kv, const int32_t* page_table,
                                                                  const int32_t* seq_lens, const uint16_t* Wcat,
                                                                  uint16_t* pool2, int32_t* table2, int32_t* lens2,
                                                                  int heads, int num_pages, int max_pages)
{
    constexpr int ROW = D_C + 64;
    constexpr int NKS = D_C / 32;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int pg = blockIdx.x, bh = blockIdx.y;
    const int b = bh / heads, h = bh % heads;
    const int L = max(0, min(seq_lens[b], max_pages * 64));
    if (pg == 0 && tid == 0) lens2[bh] = L;
    if (pg * 64 >= L) return;
    const int page = page_table[(size_t)b * max_pages + pg];
    const bool valid = page >= 0 && page < num_pages;
    // the pseudo-sequence (b, h) owns pages [bh * max_pages, +max_pages) of the materialised pool;
    // a page id outside the cache pool is passed on as "skip these tokens"
    const size_t page2 = (size_t)bh * max_pages + pg;
    if (tid == 0) table2[page2] = valid ? (int32_t)page2 : -1;
    if (!valid) return;
    const uint16_t* src = kv + (size_t)page * 64 * ROW;
    uint16_t* dst = pool2 + page2 * 64 * PF_ROW;

    // decoupled-rope part of the key: copied as it is
    for (int i = tid; i < 64 * 8; i += 256) {
        const int tok = i >> 3, ch = i & 7;
        *reinterpret_cast<u32x4*>(dst + tok * PF_ROW + PF_DH + ch * 8) =
            *reinterpret_cast<const u32x4*>(src + tok * ROW + D_C + ch * 8);
    }
    // B operand: latent row of token 16 wave + n, k = 32 ks + 8g .. + 7
    bf16x8 cb[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
        cb[ks] = *reinterpret_cast<const bf16x8*>(src + (wave * 16 + n) * ROW + ks * 32 + g * 8);
    const uint16_t* W = Wcat + (size_t)h * 256 * D_C;
    uint16_t* out_row = dst + (wave * 16 + n) * PF_ROW;
#pragma unroll 2
    for (int mt = 0; mt < 16; ++mt) {
        f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(W + (size_t)(mt * 16 + n) * D_C + ks * 32 + g * 8);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, cb[ks], acc, 0, 0, 0);
        }
        // D: rows 4g .. 4g+3 of row tile mt (output dimensions), column n (token)
        const int col = mt < 8 ? mt * 16 + g * 4 : PF_DH + 64 + (mt - 8) * 16 + g * 4;
        *reinterpret_cast<u32x2*>(out_row + col) = (u32x2){pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3])};
    }
}

}  // namespace

bool prefill_supported(int d_head, int d_c, int d_rope, int page_size, mla_dtype io, mla_dtype cache)
{
    return io == MLA_BF16 && cache == MLA_BF16 && d_head == PF_DH && d_rope == 64 && page_size == 64 &&
           (d_c == 256 || d_c == 512);
}

hipError_t launch_prefill_materialise(const void* kv, const int32_t* page_table, const int32_t* seq_lens,
                                      const void* W_UK, const void* W_UV, void* Wcat, void* pool2, int32_t* table2,
                                      int32_t* lens2, int B, int heads, int d_c, int num_pages, int max_pages,
                                      hipStream_t s)
{
    prefill_weights_kernel<<<dim3(256, heads), 256, 0, s>>>(static_cast<const uint16_t*>(W_UK),
                                                           static_cast<const uint16_t*>(W_UV),
                                                           static_cast<uint16_t*>(Wcat), d_c);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid(max_pages, B * heads);
    if (d_c == 512)
        prefill_materialise_kernel<512><<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(kv), page_table, seq_lens,
                                                             static_cast<const uint16_t*>(Wcat), static_cast<uint16_t*>(pool2),
                                                             table2, lens2, heads, num_pages, max_pages);
    else
        prefill_materialise_kernel<256><<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(kv), page_table, seq_lens,
                                                             static_cast<const uint16_t*>(Wcat), static_cast<uint16_t*>(pool2),
                                                             table2, lens2, heads, num_pages, max_pages);
    return hipGetLastError();
}

}  // namespace mla
