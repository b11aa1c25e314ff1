// What this GPU sustains on the two resources the backward-data path is measured against: HBM bytes per second with a
// plain streaming kernel, and matrix-core operations per second with the two instructions the kernels use, issued
// from registers only.  Measurement aids: the benchmark reports its roofline fractions against the published peaks
// and, beside them, against these.
#include "bwd_tiled.h"

namespace sdgp {

namespace {

constexpr int kProbeBlock = 256;

// dst[i] = src[i], 16 bytes per lane and step, streaming hints on both sides.
__global__ void __launch_bounds__(kProbeBlock) probe_copy(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst, size_t nvec) {
    const size_t stride = (size_t)gridDim.x * kProbeBlock * 4;
    for (size_t i = (size_t)blockIdx.x * kProbeBlock * 4 + threadIdx.x; i < nvec; i += stride) {
        u32x4_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + (size_t)u * kProbeBlock < nvec) v[u] = __builtin_nontemporal_load(src + i + (size_t)u * kProbeBlock);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + (size_t)u * kProbeBlock < nvec) __builtin_nontemporal_store(v[u], dst + i + (size_t)u * kProbeBlock);
    }
}

// Reads src once; every workgroup leaves one word (the xor of what it read) in sink[blockIdx.x].
__global__ void __launch_bounds__(kProbeBlock) probe_read(const u32x4_t* __restrict__ src, size_t nvec, uint32_t* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * kProbeBlock * 4;
    uint32_t acc = 0;
    for (size_t i = (size_t)blockIdx.x * kProbeBlock * 4 + threadIdx.x; i < nvec; i += stride) {
        u32x4_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            v[u] = u32x4_t{0u, 0u, 0u, 0u};
            if (i + (size_t)u * kProbeBlock < nvec) v[u] = __builtin_nontemporal_load(src + i + (size_t)u * kProbeBlock);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    __shared__ uint32_t part[kProbeBlock];
    part[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t x = 0;
        for (int i = 0; i < kProbeBlock; ++i) x ^= part[i];
        sink[blockIdx.x] = x;
    }
}

// `iters` rounds of eight independent matrix instructions per wavefront (eight accumulator tiles, so no instruction
// waits for the one before it); operands never leave the registers.  SPARSE: the structured-sparse instruction.
template <bool SPARSE>
__global__ void __launch_bounds__(kProbeBlock) probe_mfma(int iters, float* __restrict__ sink) {
    f32x16_t acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
    bf16x8_t a;
    typename std::conditional<SPARSE, bf16x16_t, bf16x8_t>::type b;
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = (__bf16)(float)((threadIdx.x + e) & 3);
#pragma unroll
    for (int e = 0; e < (SPARSE ? 16 : 8); ++e) b[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 1);
    const int meta = 0x4444;   // positions 0 and 1 of every quad
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if constexpr (SPARSE) acc[t] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a, b, acc[t], meta, 0, 0);
            else acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[t][r];
    if (s == -1.0f) sink[0] = s;   // (sums of non-negative products: never true; keeps the loop alive)
}

int probe_grid(int per_cu) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -1;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return -1;
    return cus * per_cu;
}

}  // namespace

// kind 0: copy `bytes` from a to b; 1: read `bytes` of a, b takes one word per workgroup (at most 16 KB);
// 2 / 3: `iters` rounds of eight dense / structured-sparse bf16 matrix instructions per wavefront, two wavefronts per
// SIMD, b takes nothing (it must still be a valid pointer).  Returns the work of the launch through *work: bytes
// moved (2 * bytes for the copy) or dense-equivalent floating-point operations.
int peak_probe_launch(int kind, const void* a, void* b, size_t bytes, int iters, double* work, hipStream_t stream) {
    if (kind == 0 || kind == 1) {
        const size_t nvec = bytes / 16;
        const int grid = probe_grid(16);
        if (grid <= 0) return SDGP_ERR_HIP;
        if (nvec == 0) { *work = 0.0; return SDGP_OK; }
        if (kind == 0) hipLaunchKernelGGL(probe_copy, dim3(grid), dim3(kProbeBlock), 0, stream, static_cast<const u32x4_t*>(a), static_cast<u32x4_t*>(b), nvec);
        else hipLaunchKernelGGL(probe_read, dim3(grid), dim3(kProbeBlock), 0, stream, static_cast<const u32x4_t*>(a), nvec, static_cast<uint32_t*>(b));
        *work = (kind == 0 ? 2.0 : 1.0) * 16.0 * (double)nvec;
        return launch_status();
    }
    const int grid = probe_grid(2);
    if (grid <= 0) return SDGP_ERR_HIP;
    if (kind == 2) hipLaunchKernelGGL(probe_mfma<false>, dim3(grid), dim3(kProbeBlock), 0, stream, iters, static_cast<float*>(b));
    else hipLaunchKernelGGL(probe_mfma<true>, dim3(grid), dim3(kProbeBlock), 0, stream, iters, static_cast<float*>(b));
    const double per_instr = kind == 2 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 32;
    *work = (double)grid * (kProbeBlock / 64) * (double)iters * 8.0 * per_instr;
    return launch_status();
}

}  // namespace sdgp
