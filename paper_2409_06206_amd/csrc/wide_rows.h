// Rows of one 8x8 window brought into LDS by direct loads, shared by the wide-layer kernels.
#pragma once
#include "common.h"
#include "mfma.h"

namespace gswa {

template <int C> struct WindowRows {
    static constexpr int M = 8;
    static constexpr int CHUNKS = 64 * 2 * C / 16;     // 16-byte pieces of a window's 64 rows
    static constexpr int ROW_CHUNKS = 8 * 2 * C / 16;  // of one image row of the window (8 tokens)
    static constexpr int INSTR = (CHUNKS + 63) / 64;   // load instructions per window (64 pieces each)
    // a few bytes of slack behind the last row, where operand reads of a zero-padded last K step reach
    static constexpr size_t BYTES = (size_t)CHUNKS * 16 + 64;
    static_assert((8 * 2 * C) % 16 == 0, "an image row of a window is whole 16-byte pieces");
    static_assert(ROW_CHUNKS >= 64, "fetch_window_rows advances at most one image row per instruction");
};

// The rows [64 tokens][C] (bf16) of window `win` of tensor `base` -> `stage`, in memory order: 8 image
// rows of 8 tokens, token (r, c) of the window at byte (8 r + c) 2 C.  An image row of the window is
// one contiguous run of 16 C bytes, or two in the last window column of a shifted layer, split at
// token M - shift: a whole number of 16-byte pieces because the shift is even.  Piece 64 k + lane is
// moved by the wave's instruction k; `base` must be 16-byte aligned.  Asynchronous (lds_dma16).
template <int C>
__device__ __forceinline__ void fetch_window_rows(const Geom &g, const void *base, int win, int lane, uint8_t *stage)
{
    using R = WindowRows<C>;
    constexpr int M = R::M;
    const int per_img = g.nwi * g.nwj;
    const int s = g.shift;
    const int b = win / per_img;
    const int wr = win - b * per_img;
    const int wi = wr / g.nwj, wj = wr - wi * g.nwj;
    const bool wrap = s > 0 && wj == g.nwj - 1;
    const uint32_t col_a = (uint32_t)(wj * M + s) * (2u * C);                 // first run: from this column
    const uint32_t split = wrap ? (uint32_t)(M - s) * (2u * C) : 0xffffffffu; // second run (from column 0) starts here
    const int si0 = wi * M + s;
    int cc = lane, r = 0; // piece within the image row, image row
#pragma unroll
    for (int k = 0; k < R::INSTR; ++k) {
        if (cc >= R::ROW_CHUNKS) {
            cc -= R::ROW_CHUNKS;
            ++r;
        }
        if (64 * k + lane < R::CHUNKS) {
            int si = si0 + r;
            if (si >= g.H) si -= g.H;
            const uint32_t br = 16u * cc;
            const uint32_t off = (uint32_t)((b * g.H + si) * g.W) * (2u * C) + (br < split ? col_a + br : br - split);
            lds_dma16(static_cast<const uint8_t *>(base) + off, stage + k * 1024);
        }
        cc += 64;
    }
}

} // namespace gswa
