// Optional per-kernel timing with HIP events (off by default).  When enabled, every kernel
// the library enqueues is bracketed by two events recorded on the kernel's own stream;
// gswa_profile_collect() turns them into per-kernel totals.
#pragma once
#include <hip/hip_runtime.h>

namespace gswa {

enum KernelId {
    K_FILL = 0,
    K_QKV_LINEAR,   // q|k|v projection of one group (Eq. 6), cascade add fused (Eq. 8)
    K_ATTN_FWD,     // attention core of one group
    K_PROJ_LINEAR,  // output projection (Eq. 7)
    K_PROJ_WGRAD,   // d w_proj, d b_proj
    K_DO_LINEAR,    // dO of one group = dy Wproj slice (+ cascade gradient)
    K_ATTN_BWD,     // adjoint of the attention core of one group
    K_DX_LINEAR,    // dF of one group = dqkv Wqkv
    K_QKV_WGRAD,    // d w_qkv, d b_qkv of one group
    K_PACK_FWD,     // parameters into MFMA fragment order (once per forward call, both passes use it)
    K_FUSED_FWD,    // whole forward layer, one launch
    K_FUSED_BWD,    // dx and partial parameter gradients of one head chunk
    K_REDUCE,       // per-workgroup partial sums -> parameter gradients
    K_ATTN_CHUNK_FWD, // split forward: attention of one head chunk
    K_PROJ_GEMM,    // split forward: output projection (Eq. 7)
    K_WPROJ_GRAD,   // split backward: d w_proj, d b_proj
    K_ATTN_CORE_FWD, // attention core of one group on the matrix cores
    K_ATTN_CORE_BWD, // its adjoint
    K_LINEAR_PAIR,  // backward of one group: q|k|v recomputation and dO in one launch
    K_WINDOW_FWD,   // whole forward of a narrow layer with 64- or 144-token windows, one launch
    K_LN_FWD,       // LayerNorm of every token (Eq. 4-5), optionally of a sum that is stored as well
    K_LN_BWD,       // its adjoint, skip gradient added
    K_GELU_FWD,     // hidden layer of the MLP from its pre-activation
    K_GELU_BWD,     // gradient through the GELU
    K_FC1_LINEAR,   // first fully connected layer of the MLP (Eq. 5)
    K_FC2_LINEAR,   // second one, skip connection added
    K_FC_DLINEAR,   // gradient with respect to the input of a fully connected layer
    K_FC_WGRAD,     // gradient of its weight and bias
    K_MLP_FWD,      // skip of Eq. 4 and all of Eq. 5 in one launch
    K_MLP_BWD,      // adjoint of Eq. 5 in one launch
    K_MLP_PACK,     // the MLP's weights into MFMA fragment order (once per forward call)
    K_MLP_REDUCE,   // per-workgroup partial weight gradients of the MLP -> gradients
    K_LN_FWD_REDUCE, // LayerNorm of every token and that sum in one launch
    K_WIDE_ATTN_BWD, // wide layers: adjoint of one group's attention, one wavefront per window
    K_WIDE_WGRAD,    // wide layers: a group's dx slice and weight gradients from d(q|k|v)
    K_COUNT
};

const char *kernel_name(int id);

// RAII bracket around one launch.
struct KernelTimer {
    KernelTimer(int id, hipStream_t s);
    ~KernelTimer();
    int slot;
    hipStream_t stream;
};

} // namespace gswa
