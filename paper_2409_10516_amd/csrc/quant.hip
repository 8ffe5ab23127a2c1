// 8-bit copy of the keys for the graph search. Appendix C of the paper names 8-bit scalar
// quantisation of the KV vectors as the next step without giving a scheme; the one here is
// symmetric, linear, per (sequence, KV head) and per dimension:
//     scale[d] = max_i |k[i][d]| / 127   (1 for an all-zero column)
//     k8[i][d] = clamp(round_half_even(k[i][d] / scale[d]), -127, 127)
// in float32, every division rounded once, so the bytes are reproducible on a CPU. Only the
// search reads the copy; attention uses the original keys.
#include "common.h"

#define QZ_THREADS 256
#define QZ_ROWS 64                 // rows a workgroup folds into the column maxima

template <int DT>
__device__ __forceinline__ float qz_key(const void* K, size_t i) {
    if (DT == RA_BF16) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(K)[i] << 16);
    return reinterpret_cast<const float*>(K)[i];
}

// grid (row chunks, groups); |x| of a float is monotone in its bit pattern, so the column
// maxima are taken with integer atomic-max on the bits (maxabs zeroed beforehand)
template <int DT>
__global__ __launch_bounds__(QZ_THREADS) void qz_maxabs_kernel(const void* __restrict__ K, int64_t N,
                                                               uint32_t* __restrict__ maxabs) {
    const int d = threadIdx.x % RA_D, sub = threadIdx.x / RA_D;            // two rows per pass
    const size_t g = blockIdx.y;
    const int64_t r0 = (int64_t)blockIdx.x * QZ_ROWS;
    uint32_t m = 0u;
    for (int64_t r = r0 + sub; r < r0 + QZ_ROWS && r < N; r += QZ_THREADS / RA_D) {
        const uint32_t b = __float_as_uint(qz_key<DT>(K, (g * N + r) * RA_D + d)) & 0x7fffffffu;
        m = b > m ? b : m;
    }
    if (m) atomicMax(&maxabs[g * RA_D + d], m);
}

__global__ void qz_scale_kernel(float* __restrict__ scale, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float m = scale[i];                                               // the maximum's bits are its value
    scale[i] = m == 0.f ? 1.f : __fdiv_rn(m, 127.f);
}

template <int DT>
__global__ __launch_bounds__(QZ_THREADS) void qz_write_kernel(const void* __restrict__ K, int64_t N,
                                                              const float* __restrict__ scale,
                                                              int8_t* __restrict__ K8) {
    const size_t g = blockIdx.y;
    const size_t per_group = (size_t)N * RA_D;
    for (size_t i = (size_t)blockIdx.x * QZ_THREADS + threadIdx.x; i < per_group;
         i += (size_t)gridDim.x * QZ_THREADS) {
        const float k = qz_key<DT>(K, g * per_group + i);
        float r = rintf(__fdiv_rn(k, scale[g * RA_D + i % RA_D]));         // rintf: half to even
        r = fminf(fmaxf(r, -127.f), 127.f);
        K8[g * per_group + i] = (int8_t)(int)r;
    }
}

__global__ void qz_zero_kernel(uint32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// K [n_groups][N][128] -> K8 [n_groups][N][128], scale [n_groups][128]
ra_status ra_launch_quantize(const void* K, ra_dtype dt, int n_groups, int64_t N, hipStream_t st,
                             int8_t* K8, float* scale) {
    const int ns = n_groups * RA_D;
    hipLaunchKernelGGL(qz_zero_kernel, dim3((ns + 255) / 256), dim3(256), 0, st,
                       reinterpret_cast<uint32_t*>(scale), ns);
    const dim3 g1((unsigned)((N + QZ_ROWS - 1) / QZ_ROWS), (unsigned)n_groups);
    int64_t blocks = (N * RA_D + QZ_THREADS - 1) / QZ_THREADS;
    if (blocks > 4096) blocks = 4096;
    const dim3 g2((unsigned)blocks, (unsigned)n_groups);
    if (dt == RA_BF16) {
        hipLaunchKernelGGL(qz_maxabs_kernel<RA_BF16>, g1, dim3(QZ_THREADS), 0, st, K, N,
                           reinterpret_cast<uint32_t*>(scale));
        hipLaunchKernelGGL(qz_scale_kernel, dim3((ns + 255) / 256), dim3(256), 0, st, scale, ns);
        hipLaunchKernelGGL(qz_write_kernel<RA_BF16>, g2, dim3(QZ_THREADS), 0, st, K, N, scale, K8);
    } else {
        hipLaunchKernelGGL(qz_maxabs_kernel<RA_F32>, g1, dim3(QZ_THREADS), 0, st, K, N,
                           reinterpret_cast<uint32_t*>(scale));
        hipLaunchKernelGGL(qz_scale_kernel, dim3((ns + 255) / 256), dim3(256), 0, st, scale, ns);
        hipLaunchKernelGGL(qz_write_kernel<RA_F32>, g2, dim3(QZ_THREADS), 0, st, K, N, scale, K8);
    }
    RA_HIP(hipGetLastError());
    return RA_OK;
}
