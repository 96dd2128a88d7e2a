// Shared device/host definitions of the GSWA HIP library: element types, the shift/partition
// index map and the validated layer geometry.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gswa {

// bfloat16 storage: the upper half of an fp32 pattern.
struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float(uint32_t(v.bits) << 16); }

// fp32 -> bf16, round to nearest even (NaN kept quiet).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return uint16_t(u >> 16);
}

__device__ __forceinline__ void from_f32(float &dst, float v) { dst = v; }
__device__ __forceinline__ void from_f32(bf16_t &dst, float v) { dst.bits = f32_to_bf16_bits(v); }

// Geometry of one layer call, filled by the host after validation (Sec. "Patch Embedding",
// Sec. "Group Shifted Window Attention").
struct Geom {
    int B, H, W, C;
    int heads, groups, M, shift;
    int N;        // tokens per window, M*M
    int Cg;       // channels per group
    int hg;       // heads per group
    int d;        // head width (of v and of the head's output)
    int dq;       // channels of q and of k per head (Sec. "Parameter Allocation"; d for the plain layer)
    int Qg;       // channels of q (and of k) per group, hg * dq
    int Rg;       // features a group projects to, [q: Qg | k: Qg | v: Cg]
    int nwi, nwj; // windows along H and W
    int nW;       // windows in the batch
    long T;       // tokens in the batch
    int cascade;  // Eq. 8 on/off
};

// Window w = (b, wi, wj) and in-window token n = r*M + c  ->  flat token index of x / y, and
// the id of the mask region the token belongs to (tokens of different regions were brought
// together by the cyclic shift and do not attend to each other).
__device__ __forceinline__ long window_token(const Geom &g, int w, int n, int &region)
{
    const int per_img = g.nwi * g.nwj;
    const int b = w / per_img;
    const int wr = w - b * per_img;
    const int wi = wr / g.nwj, wj = wr - wi * g.nwj;
    const int r = n / g.M, c = n - r * g.M;
    const int i = wi * g.M + r, j = wj * g.M + c;
    int si = i + g.shift, sj = j + g.shift;
    if (si >= g.H) si -= g.H;
    if (sj >= g.W) sj -= g.W;
    region = 0;
    if (g.shift > 0) {
        const int bi = i < g.H - g.M ? 0 : (i < g.H - g.shift ? 1 : 2);
        const int bj = j < g.W - g.M ? 0 : (j < g.W - g.shift ? 1 : 2);
        region = 3 * bi + bj;
    }
    return ((long)b * g.H + si) * g.W + sj;
}

// Records the text of a failed HIP call for gswa_last_hip_error() and returns GSWA_EHIP.
int report_hip_error(hipError_t e);

// Raises a kernel's limit of dynamic LDS to at least `bytes` on the current device (nothing to do up to the
// 64 KB every kernel may use).  Remembered per kernel and device, safe to call from several host threads.
hipError_t allow_dynamic_lds(const void *kernel, size_t bytes);

// Compute units of the current device, for sizing launch grids (looked up once per process, in a
// thread-safe way; 256 if the runtime cannot tell).  Buffer sizes never depend on it.
inline int device_cu_count()
{
    static const int cus = [] {
        int dev = 0, n = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) n = prop.multiProcessorCount;
        return n > 0 ? n : 256;
    }();
    return cus;
}
// The compute units every scratch size is computed for: launches use at most this many.
constexpr int kSizingCus = 256;

} // namespace gswa
