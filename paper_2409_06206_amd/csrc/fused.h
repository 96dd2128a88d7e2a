// Fused per-window GSWA kernels (bf16 storage, MFMA arithmetic, 8x8 windows).
//
// One workgroup of four wavefronts owns one window at a time; wave w owns the 16 tokens of
// window rows 2w and 2w+1 through the whole layer.  Activations stay in registers in MFMA
// operand / result layouts (see mfma.h); only K and V of a head cross waves, through LDS.
// The shift, the window partition and their inverses are the address computation of the
// first load and the last store (Sec. "Patch Embedding", Sec. "Group Shifted Window Attention").
#pragma once
#include "common.h"
#include "profile.h"

namespace gswa {

// Compile-time shape of a fused instantiation.
template <int C_, int HEADS_, int G_> struct FusedCfg {
    static constexpr int C = C_, HEADS = HEADS_, G = G_;
    static constexpr int D = C / HEADS, CG = C / G, HG = HEADS / G;
    static constexpr int ET = (D + 15) / 16;  // 16-row tiles per head (head width padded to 16*ET)
    static constexpr int KS = (CG + 31) / 32; // K=32 steps over one group's input channels
    static constexpr int OT = (C + 15) / 16;  // 16-row tiles of the output projection
    // weight fragments, stored lane-major so that one LDS read per lane fetches an MFMA operand
    static constexpr int N_WQ = HEADS * 3 * ET * KS;           // Wqkv on the x slice, K=32 fragments
    static constexpr int N_WC = (G - 1) * HG * 3 * ET * HG * ET; // Wqkv on the cascade input, K=16
    static constexpr int N_WP = OT * HEADS * ET;               // Wproj, K=16 fragments
    static constexpr size_t OFF_WQ = 0;
    static constexpr size_t OFF_WC = OFF_WQ + (size_t)N_WQ * 1024;
    static constexpr size_t OFF_WP = OFF_WC + (size_t)N_WC * 512;
    static constexpr size_t OFF_BIAS = OFF_WP + (size_t)N_WP * 512; // fp32 b_qkv [3C], b_proj [C]
    static constexpr size_t PACK_BYTES = OFF_BIAS + (size_t)16 * C;
    // per-head K and V exchange buffers, double buffered
    static constexpr int VT_LD = 68;
    static constexpr size_t OFF_K = PACK_BYTES;
    static constexpr size_t K_BYTES = (size_t)2 * 4 * ET * 64 * 8;
    static constexpr size_t OFF_VT = OFF_K + K_BYTES;
    static constexpr size_t VT_BYTES = (size_t)2 * 16 * ET * VT_LD * 2;
    static constexpr size_t FWD_LDS_BYTES = OFF_VT + VT_BYTES;
};

// True when a fused forward instantiation exists for this geometry (bf16 only).
bool fused_fwd_supported(const Geom &g);
// Bytes of scratch the fused forward needs (fragment-ordered copy of the weights).
size_t fused_fwd_ws_bytes(const Geom &g);

// y = GSWA(x); attn_out (may be null) receives the concatenated group outputs [T, C].
hipError_t launch_fused_fwd(const Geom &g, const bf16_t *x, const bf16_t *w_qkv, const bf16_t *b_qkv,
                            const bf16_t *w_proj, const bf16_t *b_proj, const bf16_t *table,
                            bf16_t *y, bf16_t *attn_out, void *ws, hipStream_t s);

bool fused_bwd_supported(const Geom &g);
// Scratch of the fused backward: packed weights + per-workgroup partial parameter gradients.
size_t fused_bwd_ws_bytes(const Geom &g);

// dx and the five parameter gradients from x, dy and the saved group outputs.  The parameter
// gradients are summed over per-workgroup partials in a fixed order (run-to-run identical) and
// overwrite their outputs unless `accumulate`.
hipError_t launch_fused_bwd(const Geom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *attn,
                            const bf16_t *w_qkv, const bf16_t *b_qkv, const bf16_t *w_proj,
                            const bf16_t *table, bf16_t *dx, float *dw_qkv, float *db_qkv, float *dw_proj,
                            float *db_proj, float *dtable, int accumulate, void *ws, hipStream_t s);

} // namespace gswa
