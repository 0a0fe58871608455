// Measurement aid for bench.py, not part of the adapter path: plain streaming kernels with the byte split of
// lordba_forward (read x, read y_base, write y_out), used as the practical HBM ceiling next to the adapter kernel and
// as the known-size reference that scales the rocprofv3 FETCH_SIZE / WRITE_SIZE counters.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

// c[i] = a[i] ^ b[i] over 16-byte units; a and b may have different lengths (c has b's length).  Streaming hints as in
// the adapter kernel.  The surplus of a (if any) is read and folded into a value that is stored only if it equals a
// run-time argument (in practice never), so the compiler cannot drop the reads.
__global__ __launch_bounds__(256) void stream_xor_kernel(const u4* __restrict__ a, const u4* __restrict__ b, u4* __restrict__ c,
                                                        int64_t na, int64_t nb, uint32_t never) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    const int64_t i0 = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    for (int64_t i = i0; i < nb; i += stride) {
        u4 v = __builtin_nontemporal_load(b + i);
        if (i < na) v ^= __builtin_nontemporal_load(a + i);
        __builtin_nontemporal_store(v, c + i);
    }
    if (na > nb) {
        u4 acc = {1u, 2u, 3u, 4u};
        for (int64_t i = nb + i0; i < na; i += stride) acc ^= __builtin_nontemporal_load(a + i);
        if ((acc[0] + acc[1] + acc[2] + acc[3]) == never) c[i0 % nb] = acc;
    }
}

__global__ __launch_bounds__(256) void copy_kernel(const u4* __restrict__ src, u4* __restrict__ dst, int64_t n) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__global__ void empty_kernel() {}
}  // namespace

// One workgroup that does nothing: the launch-to-launch floor of the stream that small calls are compared with.
extern "C" int lordba_bench_empty(void* stream) {
    hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream));
    return static_cast<int>(hipGetLastError());
}

// All pointers: device memory, 16-byte aligned; sizes in bytes, multiples of 16.  Returns 0 or the hipError_t value.
extern "C" int lordba_bench_stream(const void* a, const void* b, void* c, int64_t a_bytes, int64_t b_bytes, void* stream) {
    if (!a || !b || !c || a_bytes < 0 || b_bytes < 16 || (a_bytes & 15) || (b_bytes & 15)) return -1;
    hipLaunchKernelGGL(stream_xor_kernel, dim3(2048), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<const u4*>(a),
                       static_cast<const u4*>(b), static_cast<u4*>(c), a_bytes / 16, b_bytes / 16, 0x9e3779b9u);
    return static_cast<int>(hipGetLastError());
}

extern "C" int lordba_bench_copy(const void* src, void* dst, int64_t bytes, void* stream) {
    if (!src || !dst || bytes < 16 || (bytes & 15)) return -1;
    hipLaunchKernelGGL(copy_kernel, dim3(2048), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<const u4*>(src),
                       static_cast<u4*>(dst), bytes / 16);
    return static_cast<int>(hipGetLastError());
}
