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

// Rows with given labels -> corrected rows, out = g[a] x + b[a] (g, b: fp32 with the blending coefficient folded in),
// stored in the type of the rows or, for fp32 rows, as bfloat16.  One wave per row.  WIDE: 16-byte loads of the row,
// four groups of a lane requested before the first is used.  For the shapes the fused inference kernels do not take
// (no instance of the row-tile kernel; more than 128 clusters ranked by two launches).
template <typename TI, typename TO, bool WIDE>
__global__ __launch_bounds__(256) void k_affine_by_labels(const TI* __restrict__ x, const int32_t* __restrict__ assign, int64_t N,
                                                          int64_t D, const float* __restrict__ g, const float* __restrict__ b,
                                                          TO* __restrict__ out) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t row = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (row >= N) return;
    const int a = assign[row];
    const float* gr = g + (int64_t)a * D;
    const float* br = b + (int64_t)a * D;
    const TI* xr = x + row * D;
    TO* orow = out + row * D;
    if (WIDE) {
        constexpr int EPL = (int)(16 / sizeof(TI));  // channels per 16-byte group of the row
        constexpr int U = sizeof(TI) == 4 ? 4 : 2;   // groups per lane in flight
        for (int64_t j0 = (int64_t)lane * EPL; j0 < D; j0 += (int64_t)U * kWave * EPL) {
            uint4 xv[U];
            float4 gv[U][EPL / 4], bv[U][EPL / 4];
            int64_t j[U];
#pragma unroll
            for (int u = 0; u < U; u++) {
                const int64_t jj = j0 + (int64_t)u * kWave * EPL;
                j[u] = jj < D ? jj : j0;
                xv[u] = *(const uint4*)(xr + j[u]);
#pragma unroll
                for (int h = 0; h < EPL / 4; h++) {
                    gv[u][h] = *(const float4*)(gr + j[u] + 4 * h);
                    bv[u][h] = *(const float4*)(br + j[u] + 4 * h);
                }
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                if (j0 + (int64_t)u * kWave * EPL >= D) break;
                float v[EPL], r[EPL];
                const uint32_t w[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    if (sizeof(TI) == 4) {
                        v[e % EPL] = __uint_as_float(w[e]);
                    } else {
                        v[(2 * e) % EPL] = __uint_as_float(w[e] << 16);
                        v[(2 * e + 1) % EPL] = __uint_as_float(w[e] & 0xFFFF0000u);
                    }
                }
#pragma unroll
                for (int e = 0; e < EPL; e++) {
                    const float4 gg = gv[u][e / 4], bb = bv[u][e / 4];
                    const float ge = e % 4 == 0 ? gg.x : e % 4 == 1 ? gg.y : e % 4 == 2 ? gg.z : gg.w;
                    const float be = e % 4 == 0 ? bb.x : e % 4 == 1 ? bb.y : e % 4 == 2 ? bb.z : bb.w;
                    r[e] = fmaf(ge, v[e], be);
                }
                if (sizeof(TO) == 4) {  // fp32 rows, fp32 out
                    *(uint4*)(orow + j[u]) = make_uint4(__float_as_uint(r[0]), __float_as_uint(r[1]), __float_as_uint(r[2 % EPL]),
                                                        __float_as_uint(r[3 % EPL]));
                } else {
                    uint32_t o[EPL / 2];
#pragma unroll
                    for (int e = 0; e < EPL / 2; e++) o[e] = (uint32_t)f32_to_bf16(r[2 * e]) | ((uint32_t)f32_to_bf16(r[2 * e + 1]) << 16);
                    if (EPL == 4)
                        *(uint2*)(orow + j[u]) = make_uint2(o[0], o[1]);
                    else
                        *(uint4*)(orow + j[u]) = make_uint4(o[0], o[1], o[2 % (EPL / 2)], o[3 % (EPL / 2)]);
                }
            }
        }
    } else {
        for (int64_t j = lane; j < D; j += kWave) st_elem(orow + j, fmaf(gr[j], ld_elem(xr + j), br[j]));
    }
}
cat_status launch_affine_by_labels(const void* x, cat_dtype dt, const int32_t* assign, int64_t N, int64_t D, const float* g,
                                   const float* b, void* out, bool out_bf16, hipStream_t st) {
    dim3 grid((unsigned)((N + 3) / 4)), block(256);
    const size_t esz = dt == CAT_F32 ? 4 : 2;
    const bool wide = (D * esz) % 16 == 0 && D % 4 == 0 &&
                      (((uintptr_t)x | (uintptr_t)g | (uintptr_t)b | (uintptr_t)out) & 15u) == 0;
#define CAT_AL(TI, TO, W) hipLaunchKernelGGL((k_affine_by_labels<TI, TO, W>), grid, block, 0, st, (const TI*)x, assign, N, D, g, b, (TO*)out)
    if (dt == CAT_BF16) {
        if (wide) CAT_AL(bf16_t, bf16_t, true); else CAT_AL(bf16_t, bf16_t, false);
    } else if (out_bf16) {
        if (wide) CAT_AL(float, bf16_t, true); else CAT_AL(float, bf16_t, false);
    } else {
        if (wide) CAT_AL(float, float, true); else CAT_AL(float, float, false);
    }
#undef CAT_AL
    CAT_LAUNCH_CHECK("k_affine_by_labels");
    return CAT_OK;
}

}  // namespace cat
