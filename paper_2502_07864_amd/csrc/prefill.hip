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
//   prefill_materialise_kernel  one workgroup per (pair of pages, sequence, head):
//                               Y^T [256 x 128 tokens] = Wcat[h] [256 x d_c] . C^T [d_c x 128 tokens]
//                               on v_mfma_f32_16x16x32_bf16; a wavefront owns 32 tokens, keeps
//                               their latent rows in registers as the B operand and walks the 16
//                               row tiles of Wcat[h], which all four wavefronts read from LDS;
//                               rows are rounded to bf16 and stored as
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

// One workgroup = two pages (128 tokens) of one (sequence, head).  Wcat[h] is streamed through LDS
// in chunks of 32 rows (two row tiles, all d_c columns), double-buffered, rows padded by 16 bytes so
// that the 16 rows of an A read fall in different banks; the four wavefronts share every chunk.
// A wavefront owns 32 tokens (two column tiles) and keeps their latent rows in registers.
template <int D_C>
__global__ __launch_bounds__(256, 2) void prefill_materialise_kernel(const uint16_t* kv, const int32_t* page_table,
                                                                     const int32_t* seq_lens, const uint16_t* Wcat,
                                                                     uint16_t* pool2, int32_t* table2, int32_t* lens2,
                                                                     int heads, int num_pages, int max_pages)
{
    constexpr int ROW = D_C + 64;
    constexpr int NKS = D_C / 32;
    constexpr int WROWB = D_C * 2 + 16;               // padded bytes per weight row in LDS
    constexpr int CHUNK_ROWS = 32;
    constexpr int NCHUNK = 256 / CHUNK_ROWS;          // 8
    constexpr int PIECES = CHUNK_ROWS * (D_C / 8);    // 16-byte pieces per chunk (2048 / 1024)
    constexpr int NPL = PIECES / 256;                 // pieces per thread (8 / 4)
    __shared__ __attribute__((aligned(16))) unsigned char wbuf[2][CHUNK_ROWS * WROWB];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int bh = blockIdx.y;
    const int b = bh / heads, h = bh % heads;
    const int L = max(0, min(seq_lens[b], max_pages * 64));
    if (blockIdx.x == 0 && tid == 0) lens2[bh] = L;
    if (blockIdx.x * 128 >= L) return;

    // this wavefront's page (waves 0, 1: the first of the pair; 2, 3: the second)
    const int pg = blockIdx.x * 2 + (wave >> 1);
    const bool in_seq = pg < max_pages && pg * 64 < L;
    const int page = in_seq ? page_table[(size_t)b * max_pages + pg] : -1;
    const bool active = in_seq && page >= 0 && page < num_pages;
    // the pseudo-sequence (b, h) owns pages [bh * max_pages, +max_pages) of the materialised pool;
    // a page id outside the cache pool is passed on as "skip these tokens"
    const size_t page2 = (size_t)bh * max_pages + pg;
    if (in_seq && (wave & 1) == 0 && lane == 0) table2[page2] = active ? (int32_t)page2 : -1;
    const uint16_t* src = kv + (size_t)(active ? page : 0) * 64 * ROW;
    uint16_t* dst = pool2 + (active ? page2 : 0) * 64 * PF_ROW;
    const int tok0 = (wave & 1) * 32;                 // this wavefront's first token inside its page

    bf16x8 cb[2][NKS];
    if (active) {
        // decoupled-rope part of the key: copied as it is (32 tokens x 8 pieces per wavefront)
        for (int i = lane; i < 32 * 8; i += 64) {
            const int tok = tok0 + (i >> 3), ch = i & 7;
            *reinterpret_cast<u32x4*>(dst + tok * PF_ROW + PF_DH + ch * 8) =
                *reinterpret_cast<const u32x4*>(src + tok * ROW + D_C + ch * 8);
        }
        // B operands: latent rows of tokens tok0 + 16 nt + n, k = 32 ks + 8g .. + 7
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                cb[nt][ks] = *reinterpret_cast<const bf16x8*>(src + (tok0 + nt * 16 + n) * ROW + ks * 32 + g * 8);
    }

    const unsigned char* W = reinterpret_cast<const unsigned char*>(Wcat + (size_t)h * 256 * D_C);
    u32x4 stage[NPL];
    auto load_chunk = [&](int c) {
#pragma unroll
        for (int i = 0; i < NPL; ++i) {
            const int q = i * 256 + tid;
            stage[i] = *reinterpret_cast<const u32x4*>(W + ((size_t)(c * CHUNK_ROWS) * D_C + (size_t)q * 8) * 2);
        }
    };
    auto store_chunk = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NPL; ++i) {
            const int q = i * 256 + tid;
            const int row = q / (D_C / 8), col = q % (D_C / 8);
            *reinterpret_cast<u32x4*>(&wbuf[buf][row * WROWB + col * 16]) = stage[i];
        }
    };
    load_chunk(0);
    store_chunk(0);
    __syncthreads();
    for (int c = 0; c < NCHUNK; ++c) {
        if (c + 1 < NCHUNK) load_chunk(c + 1);        // in flight while this chunk is used
        if (active) {
            f32x4 acc[2][2];
#pragma unroll
            for (int ml = 0; ml < 2; ++ml)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) acc[ml][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                for (int ml = 0; ml < 2; ++ml) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8*>(&wbuf[c & 1][(ml * 16 + n) * WROWB + ks * 64 + g * 16]);
                    acc[ml][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, cb[0][ks], acc[ml][0], 0, 0, 0);
                    acc[ml][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, cb[1][ks], acc[ml][1], 0, 0, 0);
                }
            // D: rows 4g .. 4g+3 of row tile mt = 2c + ml (output dimensions), column n (token)
#pragma unroll
            for (int ml = 0; ml < 2; ++ml) {
                const int mt = c * 2 + ml;
                const int col = mt < 8 ? mt * 16 + g * 4 : PF_DH + 64 + (mt - 8) * 16 + g * 4;
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    *reinterpret_cast<u32x2*>(dst + (tok0 + nt * 16 + n) * PF_ROW + col) =
                        (u32x2){pack_bf16x2(acc[ml][nt][0], acc[ml][nt][1]), pack_bf16x2(acc[ml][nt][2], acc[ml][nt][3])};
            }
        }
        if (c + 1 < NCHUNK) store_chunk((c + 1) & 1); // the other buffer: last read before the previous barrier
        __syncthreads();
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
    dim3 grid((max_pages + 1) / 2, B * heads);
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
