// Measurement aid: LDS read throughput, the on-chip roofline of the sparse products' walk
// (one 4-byte activation operand per multiply-add comes from LDS).
#include "common.h"

namespace mst {

// W bytes per lane and read; the 64 lanes of a wavefront read 64 W consecutive bytes (no
// bank conflicts), eight independent reads per iteration
template <int W>
__global__ __launch_bounds__(1024) void k_probe_lds_read(float* __restrict__ out, int iters) {
    __shared__ float lds[16384];   // 64 KB
    for (int i = threadIdx.x; i < 16384; i += blockDim.x) lds[i] = (float)i;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const char* b = reinterpret_cast<const char*>(lds);
    float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
    unsigned off = (threadIdx.x >> 6) * 2048u;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const unsigned a = (off + u * 4096u + (unsigned)(lane * W)) & 65535u;
            if (W == 4) { const float v = *reinterpret_cast<const float*>(b + a); acc0 += v; }
            if (W == 8) { const float2 v = *reinterpret_cast<const float2*>(b + a); acc0 += v.x; acc1 += v.y; }
            if (W == 16) {
                const float4 v = *reinterpret_cast<const float4*>(b + a);
                acc0 += v.x; acc1 += v.y; acc2 += v.z; acc3 += v.w;
            }
        }
        off = (off + 512u) & 65535u;
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc0 + acc1 + acc2 + acc3;
}

}  // namespace mst

using namespace mst;

extern "C" int mst_probe_lds_read(float* out_dev, int width, int iters, int blocks, mst_stream_t stream) {
    if (!out_dev || iters < 1 || blocks < 1 || blocks > 65535) return MST_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (width == 4) k_probe_lds_read<4><<<blocks, 1024, 0, s>>>(out_dev, iters);
    else if (width == 8) k_probe_lds_read<8><<<blocks, 1024, 0, s>>>(out_dev, iters);
    else if (width == 16) k_probe_lds_read<16><<<blocks, 1024, 0, s>>>(out_dev, iters);
    else return MST_ERR_ARG;
    MST_LAUNCH_CHECK();
    return MST_OK;
}
