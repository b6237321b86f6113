// Low-precision deployment of a fitted CAT transformation: parameters stored as bfloat16, corrected rows written as
// bfloat16.  (Sec. 3.1 of the paper remarks that the clustering yields low-precision gamma and beta and gives no
// mechanism; bfloat16 storage with round-to-nearest-even is the reading taken here.)  Kernels and launchers; the
// entry points are in cat_api.hip.
#include "cat_common.h"

namespace cat {

// dst[i] = bfloat16 nearest to src[i], ties to the even significand
__global__ __launch_bounds__(256) void k_to_bf16(const float* __restrict__ src, int64_t n, bf16_t* __restrict__ dst) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = f32_to_bf16(src[i]);
}
cat_status launch_to_bf16(const float* src, int64_t n, uint16_t* dst, hipStream_t st) {
    hipLaunchKernelGGL(k_to_bf16, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, src, n, dst);
    CAT_LAUNCH_CHECK("k_to_bf16");
    return CAT_OK;
}

// Stored parameters back to the fp32 working arrays of the inference kernels, the blending coefficient folded in:
// c = centroid, g = 1 + alpha (gamma - 1), b = alpha beta  (exactly gamma, beta when alpha = 1).
__global__ __launch_bounds__(256) void k_expand_params(const bf16_t* __restrict__ cent, const bf16_t* __restrict__ gamma,
                                                       const bf16_t* __restrict__ beta, float alpha, int64_t n,
                                                       float* __restrict__ c, float* __restrict__ g, float* __restrict__ b) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    c[i] = bf16_to_f32(cent[i]);
    const float gi = bf16_to_f32(gamma[i]), bi = bf16_to_f32(beta[i]);
    g[i] = alpha == 1.0f ? gi : 1.f + alpha * (gi - 1.f);
    b[i] = alpha == 1.0f ? bi : alpha * bi;
}
cat_status launch_expand_params(const uint16_t* cent, const uint16_t* gamma, const uint16_t* beta, float alpha, int64_t n,
                                float* c, float* g, float* b, hipStream_t st) {
    hipLaunchKernelGGL(k_expand_params, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, cent, gamma, beta, alpha, n, c, g, b);
    CAT_LAUNCH_CHECK("k_expand_params");
    return CAT_OK;
}

// fp32 rows, given labels -> corrected rows in bfloat16: out = bf16(g[a] x + b[a]).  One wave per row.  WIDE: 16-byte
// loads, 8-byte stores, four groups of a lane requested before the first is used.  For the shapes the fused
// inference kernel has no instance for.
template <bool WIDE>
__global__ __launch_bounds__(256) void k_affine_to_bf16(const float* __restrict__ x, const int32_t* __restrict__ assign, int64_t N,
                                                        int64_t D, const float* __restrict__ g, const float* __restrict__ b,
                                                        bf16_t* __restrict__ out) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t row = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (row >= N) return;
    const int a = assign[row];
    const float* gr = g + (int64_t)a * D;
    const float* br = b + (int64_t)a * D;
    const float* xr = x + row * D;
    bf16_t* orow = out + row * D;
    if (WIDE) {
        constexpr int U = 4;
        for (int64_t j0 = (int64_t)lane * 4; j0 < D; j0 += (int64_t)U * kWave * 4) {
            float4 xv[U], gv[U], bv[U];
            int64_t j[U];
#pragma unroll
            for (int u = 0; u < U; u++) {
                const int64_t jj = j0 + (int64_t)u * kWave * 4;
                j[u] = jj < D ? jj : j0;
                xv[u] = *(const float4*)(xr + j[u]);
                gv[u] = *(const float4*)(gr + j[u]);
                bv[u] = *(const float4*)(br + j[u]);
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                if (j0 + (int64_t)u * kWave * 4 >= D) break;
                uint2 o;
                o.x = (uint32_t)f32_to_bf16(fmaf(gv[u].x, xv[u].x, bv[u].x)) | ((uint32_t)f32_to_bf16(fmaf(gv[u].y, xv[u].y, bv[u].y)) << 16);
                o.y = (uint32_t)f32_to_bf16(fmaf(gv[u].z, xv[u].z, bv[u].z)) | ((uint32_t)f32_to_bf16(fmaf(gv[u].w, xv[u].w, bv[u].w)) << 16);
                *(uint2*)(orow + j[u]) = o;
            }
        }
    } else {
        for (int64_t j = lane; j < D; j += kWave) orow[j] = f32_to_bf16(fmaf(gr[j], xr[j], br[j]));
    }
}
cat_status launch_affine_to_bf16(const float* x, const int32_t* assign, int64_t N, int64_t D, const float* g, const float* b,
                                 uint16_t* out, hipStream_t st) {
    dim3 grid((unsigned)((N + 3) / 4)), block(256);
    const bool wide = D % 4 == 0 && (((uintptr_t)x | (uintptr_t)g | (uintptr_t)b) & 15u) == 0 && ((uintptr_t)out & 7u) == 0;
    if (wide)
        hipLaunchKernelGGL(k_affine_to_bf16<true>, grid, block, 0, st, x, assign, N, D, g, b, out);
    else
        hipLaunchKernelGGL(k_affine_to_bf16<false>, grid, block, 0, st, x, assign, N, D, g, b, out);
    CAT_LAUNCH_CHECK("k_affine_to_bf16");
    return CAT_OK;
}

}  // namespace cat
