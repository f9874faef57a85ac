// Measurement helpers of libhag: kernels that only move bytes, in the access shape of the
// aggregation kernels, so that a benchmark run can state the ceilings its roofline fractions
// are measured against (rows served by L2, by the memory-side cache, by HBM, by LDS; a plain
// streaming copy).  They compute nothing of the method.
#include "hag_device_common.hpp"

namespace hag {

// cheap integer hash: the row a sub-group reads in step i
__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

// Every sub-group of LPR lanes reads `reads` pseudo-random rows of a [n_rows, d] fp32 matrix, four
// rows in flight, each row as one contiguous run of 16-byte loads (the gather kernel's access
// shape without its index loads), and adds them up.  n_rows must be a power of two.
//   LDS = 0: rows come from global memory; the matrix size decides which level serves them;
//   LDS = 1: the workgroup first copies rows [0, lds_rows) into LDS and reads those;
//   LDS = 2: instead of reading, every sub-group adds a row held in registers into pseudo-random
//            LDS rows of its own (rows g, g + groups, ...: no two sub-groups touch the same row) with
//            a 16-byte read, four adds and a 16-byte write: what an accumulator kept in LDS costs;
//   LDS = 3: the same with four LDS atomic adds per lane instead of the read and the write.
template <int LPR, int LDS>
__global__ __launch_bounds__(kBlock) void probe_rows_kernel(const float *__restrict__ src, uint32_t row_mask, int32_t d,
                                                            int32_t reads, int32_t lds_rows, float *__restrict__ sink) {
    extern __shared__ __align__(16) unsigned char probe_smem[];
    float *buf = reinterpret_cast<float *>(probe_smem);
    const int lane = threadIdx.x & (kWave - 1);
    const int sl = lane % LPR;
    const int q = d / 4;
    const int cb = min(sl, q - 1) * 4;
    const uint32_t group = (uint32_t)((blockIdx.x * kBlock + threadIdx.x) / LPR);
    if (LDS) {
        for (int i = threadIdx.x; i < lds_rows * q; i += kBlock)
            *reinterpret_cast<float4 *>(buf + 4 * (size_t)i) = ld4(src + 4 * (size_t)i);
        __syncthreads();
    }
    float4 acc{};
    if (LDS >= 2) {
        constexpr int kGroups = kBlock / LPR;                        // sub-groups of the workgroup
        const uint32_t own = (uint32_t)(threadIdx.x / LPR);
        const uint32_t mask = (uint32_t)(lds_rows / kGroups - 1);    // lds_rows / kGroups is a power of two >= 1
        const uint32_t row_bytes = (uint32_t)d * 4u;
        unsigned char *base = probe_smem + (uint32_t)cb * 4u;
        uint32_t a = probe_hash(group * 0x9e3779b9U + 1u);
        const float4 v = ld4(src + cb);
        for (int i = 0; i < reads; ++i) {
            a = a * 1664525u + 1013904223u;
            float *p = reinterpret_cast<float *>(base + __umul24(((a >> 16) & mask) * kGroups + own, row_bytes));
            if (LDS == 2) {
                float4 t = *reinterpret_cast<float4 *>(p);
                add4(t, v);
                *reinterpret_cast<float4 *>(p) = t;
            } else {
                __hip_atomic_fetch_add(p + 0, v.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                __hip_atomic_fetch_add(p + 1, v.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                __hip_atomic_fetch_add(p + 2, v.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                __hip_atomic_fetch_add(p + 3, v.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
        __syncthreads();
        acc = *reinterpret_cast<const float4 *>(base + __umul24(own, row_bytes));
    } else if (LDS) {
        // Row numbers come from a linear congruential sequence, two per step, and are turned into byte
        // offsets with 24-bit multiplies: a dozen vector instructions per four row reads, so that the
        // loop is limited by the LDS reads and not by the arithmetic around them.
        const uint32_t mask = (uint32_t)(lds_rows - 1);        // at most 4095
        const uint32_t row_bytes = (uint32_t)d * 4u, col_bytes = (uint32_t)cb * 4u;
        const unsigned char *base = probe_smem + col_bytes;
        uint32_t a = probe_hash(group * 0x9e3779b9U + 1u);
        for (int i = 0; i < reads; i += 4) {
            a = a * 1664525u + 1013904223u;
            const uint32_t o0 = __umul24((a >> 20) & mask, row_bytes), o1 = __umul24((a >> 8) & mask, row_bytes);
            a = a * 1664525u + 1013904223u;
            const uint32_t o2 = __umul24((a >> 20) & mask, row_bytes), o3 = __umul24((a >> 8) & mask, row_bytes);
            const float4 v0 = *reinterpret_cast<const float4 *>(base + o0);
            const float4 v1 = *reinterpret_cast<const float4 *>(base + o1);
            const float4 v2 = *reinterpret_cast<const float4 *>(base + o2);
            const float4 v3 = *reinterpret_cast<const float4 *>(base + o3);
            add4(acc, v0); add4(acc, v1); add4(acc, v2); add4(acc, v3);
        }
    } else {
        for (int i = 0; i < reads; i += 4) {
            uint32_t r[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) r[k] = probe_hash(group * 0x9e3779b9U + (uint32_t)(i + k)) & row_mask;
            float4 v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] = ld4(src + (size_t)r[k] * d + cb);
#pragma unroll
            for (int k = 0; k < 4; ++k) add4(acc, v[k]);
        }
    }
    st4(sink + 4 * ((size_t)blockIdx.x * kBlock + threadIdx.x), acc);
}

// grid-stride streaming copy, 16 bytes per lane and step
__global__ __launch_bounds__(kBlock) void probe_copy_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst,
                                                            int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// fp32 matrix-core throughput: every wavefront issues `iters` rounds of four independent
// v_mfma_f32_32x32x2_f32 (4096 flops each) on register operands; nothing but the matrix pipe is used
typedef float probe_acc_t __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(kBlock) void probe_mfma_f32_kernel(int32_t iters, float *__restrict__ sink) {
    probe_acc_t a0 = {0}, a1 = {0}, a2 = {0}, a3 = {0};
    const float x = (float)(threadIdx.x & 7) * 0.125f, y = 1.0f / (float)(1 + (threadIdx.x & 3));
    for (int i = 0; i < iters; ++i) {
        a0 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, a0, 0, 0, 0);
        a1 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, x, a1, 0, 0, 0);
        a2 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, x, a2, 0, 0, 0);
        a3 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, y, a3, 0, 0, 0);
    }
    float r = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) r += a0[k] + a1[k] + a2[k] + a3[k];
    sink[(size_t)blockIdx.x * kBlock + threadIdx.x] = r;
}

template <int LDS>
static int launch_probe_rows(int lpr, unsigned groups, size_t lds_bytes, hipStream_t s, const float *src, uint32_t mask,
                             int32_t d, int32_t reads, int32_t lds_rows, float *sink) {
    const dim3 grid(groups), block(kBlock);
    switch (lpr) {
        case 4: hipLaunchKernelGGL((probe_rows_kernel<4, LDS>), grid, block, lds_bytes, s, src, mask, d, reads, lds_rows, sink); break;
        case 8: hipLaunchKernelGGL((probe_rows_kernel<8, LDS>), grid, block, lds_bytes, s, src, mask, d, reads, lds_rows, sink); break;
        case 16: hipLaunchKernelGGL((probe_rows_kernel<16, LDS>), grid, block, lds_bytes, s, src, mask, d, reads, lds_rows, sink); break;
        case 32: hipLaunchKernelGGL((probe_rows_kernel<32, LDS>), grid, block, lds_bytes, s, src, mask, d, reads, lds_rows, sink); break;
        default: hipLaunchKernelGGL((probe_rows_kernel<64, LDS>), grid, block, lds_bytes, s, src, mask, d, reads, lds_rows, sink); break;
    }
    HIP_TRY(hipGetLastError());
    return HAG_OK;
}

}  // namespace hag

using namespace hag;

extern "C" {

int64_t hag_probe_rows(const void *src, int64_t n_rows, int64_t d, int64_t reads, int32_t from_lds, int64_t workgroups,
                       void *sink, void *stream) {
    if (!src || !sink) { set_error("NULL pointer"); return HAG_EINVAL; }
    if (((uintptr_t)src | (uintptr_t)sink) & 15) { set_error("pointers must be 16-byte aligned"); return HAG_EINVAL; }
    if (d <= 0 || d % 4 != 0 || d > 256) { set_error("d must be a multiple of 4 in [4, 256]"); return HAG_EINVAL; }
    if (n_rows <= 0 || (n_rows & (n_rows - 1)) != 0 || n_rows > (1LL << 31)) { set_error("n_rows must be a power of two"); return HAG_EINVAL; }
    if (reads <= 0 || reads % 4 != 0 || reads > (1 << 24)) { set_error("reads must be a positive multiple of 4"); return HAG_EINVAL; }
    if (workgroups <= 0 || workgroups > (1 << 20)) { set_error("workgroups out of range"); return HAG_EINVAL; }
    const int lpr = pick_lpr(d);
    const int64_t groups_per_wg = kBlock / lpr;
    int rc;
    if (from_lds < 0 || from_lds > 3) { set_error("from_lds must be 0..3"); return HAG_EINVAL; }
    if (from_lds) {
        // as many rows as fit 16 KB (so that eight workgroups share a compute unit, like the kernels
        // this stands for), a power of two, at most n_rows; the accumulating forms need a row per sub-group
        int64_t lds_rows = 1;
        while (lds_rows * 2 * d * 4 <= 16 * 1024 && lds_rows * 2 <= n_rows) lds_rows *= 2;
        if (from_lds >= 2 && lds_rows < groups_per_wg) { set_error("n_rows too small for an LDS row per sub-group"); return HAG_EINVAL; }
        const size_t lds_bytes = (size_t)(lds_rows * d * 4);
        const hipStream_t s = (hipStream_t)stream;
        const float *f = (const float *)src;
        if (from_lds == 1) rc = launch_probe_rows<1>(lpr, (unsigned)workgroups, lds_bytes, s, f, 0u, (int32_t)d, (int32_t)reads, (int32_t)lds_rows, (float *)sink);
        else if (from_lds == 2) rc = launch_probe_rows<2>(lpr, (unsigned)workgroups, lds_bytes, s, f, 0u, (int32_t)d, (int32_t)reads, (int32_t)lds_rows, (float *)sink);
        else rc = launch_probe_rows<3>(lpr, (unsigned)workgroups, lds_bytes, s, f, 0u, (int32_t)d, (int32_t)reads, (int32_t)lds_rows, (float *)sink);
    } else {
        rc = launch_probe_rows<0>(lpr, (unsigned)workgroups, 0, (hipStream_t)stream, (const float *)src,
                                  (uint32_t)(n_rows - 1), (int32_t)d, (int32_t)reads, 0, (float *)sink);
    }
    if (rc) return rc;
    return workgroups * groups_per_wg * reads * d * 4;   // bytes of rows read
}

int64_t hag_probe_mfma_f32(int64_t iters, int64_t workgroups, void *sink, void *stream) {
    if (!sink || ((uintptr_t)sink & 15)) { set_error("sink must be a 16-byte aligned device pointer"); return HAG_EINVAL; }
    if (iters <= 0 || iters > (1 << 24) || workgroups <= 0 || workgroups > (1 << 20)) { set_error("iters or workgroups out of range"); return HAG_EINVAL; }
    hipLaunchKernelGGL(probe_mfma_f32_kernel, dim3((unsigned)workgroups), dim3(kBlock), 0, (hipStream_t)stream, (int32_t)iters,
                       (float *)sink);
    HIP_TRY(hipGetLastError());
    return workgroups * (kBlock / kWave) * iters * 4 * 4096;   // flops
}

int hag_probe_copy(const void *src, void *dst, int64_t bytes, void *stream) {
    if (!src || !dst) { set_error("NULL pointer"); return HAG_EINVAL; }
    if ((((uintptr_t)src | (uintptr_t)dst) & 15) || bytes <= 0 || bytes % 16 != 0) {
        set_error("pointers and size must be multiples of 16 bytes");
        return HAG_EINVAL;
    }
    hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 16), dim3(kBlock), 0, (hipStream_t)stream, (const float4 *)src,
                       (float4 *)dst, bytes / 16);
    HIP_TRY(hipGetLastError());
    return HAG_OK;
}

}  // extern "C"
