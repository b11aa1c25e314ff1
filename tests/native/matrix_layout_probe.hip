// Test helper (not part of the library): one wavefront executes one matrix instruction, or one transposing LDS read,
// on register contents given per lane, and writes the result registers per lane.  The GPU test lays out small integer
// matrices by the operand layouts the kernels assume and checks that the result is the matrix product.
//
// Pointers are device pointers unless named host; arrays are indexed [lane][register element].  Built by the package's build step
// into tests/native/libmatrix_layout_probe.so.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16_t __attribute__((ext_vector_type(16)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x16_t __attribute__((ext_vector_type(16)));

__global__ void __launch_bounds__(64) k_mfma(const short* a, const short* b, float* d) {
    const int l = threadIdx.x;
    s16x8_t ra, rb;
    for (int e = 0; e < 8; ++e) ra[e] = a[l * 8 + e], rb[e] = b[l * 8 + e];
    f32x16_t acc = {};
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, ra), __builtin_bit_cast(bf16x8_t, rb), acc, 0, 0, 0);
    for (int r = 0; r < 16; ++r) d[l * 16 + r] = acc[r];
}

__global__ void __launch_bounds__(64) k_smfmac(const short* a, const uint32_t* idx, const short* b, float* d) {
    const int l = threadIdx.x;
    s16x8_t ra;
    s16x16_t rb;
    for (int e = 0; e < 8; ++e) ra[e] = a[l * 8 + e];
    for (int e = 0; e < 16; ++e) rb[e] = b[l * 16 + e];
    f32x16_t acc = {};
    acc = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(__builtin_bit_cast(bf16x8_t, ra), __builtin_bit_cast(bf16x16_t, rb), acc,
                                                    (int)idx[l], 0, 0);
    for (int r = 0; r < 16; ++r) d[l * 16 + r] = acc[r];
}

typedef float f32x4_t __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(64) k_mfma16(const short* a, const short* b, float* d) {
    const int l = threadIdx.x;
    s16x8_t ra, rb;
    for (int e = 0; e < 8; ++e) ra[e] = a[l * 8 + e], rb[e] = b[l * 8 + e];
    f32x4_t acc = {};
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ra), __builtin_bit_cast(bf16x8_t, rb), acc, 0, 0, 0);
    for (int r = 0; r < 4; ++r) d[l * 4 + r] = acc[r];
}

struct LaneAddr {
    uint32_t byte[64];
};

// LDS holds `words` 16-bit values copied from `in`; lane l reads four of them with the transposing read at byte
// address addr.byte[l] (checked on the host: a multiple of 8 inside the array).
__global__ void __launch_bounds__(64) k_read_tr(const short* in, int words, LaneAddr addr, short* out) {
    __shared__ __attribute__((aligned(16))) short lds[4096];
    for (int i = threadIdx.x; i < words; i += 64) lds[i] = in[i];
    __syncthreads();
    const int l = threadIdx.x;
    const s16x4_t q = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4_t*)((__attribute__((address_space(3))) char*)lds + addr.byte[l]));
    for (int e = 0; e < 4; ++e) out[l * 4 + e] = q[e];
}

}  // namespace

extern "C" {

int layout_mfma_32x32x16_bf16(const void* a, const void* b, void* d, void* stream) {
    k_mfma<<<1, 64, 0, (hipStream_t)stream>>>((const short*)a, (const short*)b, (float*)d);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int layout_mfma_16x16x32_bf16(const void* a, const void* b, void* d, void* stream) {
    k_mfma16<<<1, 64, 0, (hipStream_t)stream>>>((const short*)a, (const short*)b, (float*)d);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int layout_smfmac_32x32x32_bf16(const void* a, const void* idx, const void* b, void* d, void* stream) {
    k_smfmac<<<1, 64, 0, (hipStream_t)stream>>>((const short*)a, (const uint32_t*)idx, (const short*)b, (float*)d);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// addr_host: 64 byte addresses in HOST memory.
int layout_ds_read_tr16_b64(const void* in, int words, const uint32_t* addr_host, void* out, void* stream) {
    if (words < 4 || words > 4096 || !addr_host) return 2;
    LaneAddr addr;
    for (int l = 0; l < 64; ++l) {
        if (addr_host[l] % 8 != 0 || addr_host[l] + 8 > (uint32_t)words * 2) return 2;
        addr.byte[l] = addr_host[l];
    }
    k_read_tr<<<1, 64, 0, (hipStream_t)stream>>>((const short*)in, words, addr, (short*)out);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}
