// Binarising and packing the latent carriers on the device (training: B1 = sign(U1), B2 = sign(U2) are taken anew in
// every forward pass, Sec. 3.2 / Alg. QAT-LoRDBA).  sign(0) = +1 (Sec. 2, Notation), compared by value, so -0.0 is +1.
// One wave packs 64 consecutive bits of an output stream with one ballot; the transposed streams gather their
// entries from the same two latent arrays.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lordba.h"

namespace {

struct PackArgs {
    const float* latA;   // [r, d_in]
    const float* latB;   // [d_out, r]
    uint32_t* out[4];    // packedA [r, d_in], packedB [d_out, r], packedAt [d_in, r], packedBt [r, d_out]; may be null
    int64_t d_in, d_out, r;
    int64_t waves[4];    // waves per output stream (64 bits each)
};

__global__ __launch_bounds__(256) void lordba_pack_latents_kernel(PackArgs a) {
    const int lane = threadIdx.x & 63;
    int64_t w = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    int which = 0;
    while (which < 4 && w >= a.waves[which]) { w -= a.waves[which]; ++which; }
    if (which == 4) return;
    const int64_t n = w * 64 + lane;  // position in the row-major bit stream of the output matrix
    const int64_t nA = a.r * a.d_in, nB = a.d_out * a.r;
    const int64_t total = (which == 0 || which == 2) ? nA : nB;
    bool neg = false;
    if (n < total) {
        float u;
        if (which == 0) u = a.latA[n];
        else if (which == 1) u = a.latB[n];
        else if (which == 2) u = a.latA[(n % a.r) * a.d_in + n / a.r];      // entry (i, k) of S_A^T is entry (k, i) of S_A
        else u = a.latB[(n % a.d_out) * a.r + n / a.d_out];                 // entry (k, j) of S_B^T is entry (j, k) of S_B
        neg = u < 0.f;  // bit = 1 encodes -1; zero, -0.0 (and NaN) give +1
    }
    const uint64_t bits = __builtin_amdgcn_ballot_w64(neg);  // pad bits past the end are 0
    const int64_t nwords = (total + 31) >> 5;
    if (lane < 2 && 2 * w + lane < nwords) a.out[which][2 * w + lane] = static_cast<uint32_t>(bits >> (32 * lane));
}

}  // namespace

extern "C" lordba_status lordba_pack_latents(const float* latentA, const float* latentB,
                                             uint32_t* packedA, uint32_t* packedB, uint32_t* packedAt, uint32_t* packedBt,
                                             int64_t d_in, int64_t d_out, int64_t r, void* stream) {
    if (d_in < 1 || d_out < 1 || r < 1 || r > LORDBA_MAX_RANK || d_in > (1 << 24) || d_out > (1 << 24)) return LORDBA_ERR_DIM;
    if (!latentA || !latentB) return LORDBA_ERR_NULL;
    uint32_t* outs[4] = {packedA, packedB, packedAt, packedBt};
    if ((reinterpret_cast<uintptr_t>(latentA) | reinterpret_cast<uintptr_t>(latentB)) & 3) return LORDBA_ERR_ALIGN;
    PackArgs a;
    a.latA = latentA;
    a.latB = latentB;
    a.d_in = d_in;
    a.d_out = d_out;
    a.r = r;
    int64_t waves = 0;
    for (int i = 0; i < 4; ++i) {
        if (reinterpret_cast<uintptr_t>(outs[i]) & 3) return LORDBA_ERR_ALIGN;
        a.out[i] = outs[i];
        const int64_t bits = (i == 0 || i == 2) ? r * d_in : d_out * r;
        a.waves[i] = outs[i] ? (bits + 63) / 64 : 0;
        waves += a.waves[i];
    }
    if (waves == 0) return LORDBA_OK;
    hipLaunchKernelGGL(lordba_pack_latents_kernel, dim3(static_cast<unsigned>((waves + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), a);
    return hipGetLastError() == hipSuccess ? LORDBA_OK : LORDBA_ERR_LAUNCH;
}
