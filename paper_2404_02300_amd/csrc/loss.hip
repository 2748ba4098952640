// Softmax cross-entropy over the seed rows, the SGD update, and the library's
// error/version plumbing.
#include <stdarg.h>

#include "common.h"

namespace sdt {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

namespace {

constexpr int TB = 256;

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// One wavefront per seed row: loss_i = logsumexp(z_i) - z_i[y_i]; dZ = (softmax - onehot)/B.
// The mean of the row losses is taken later, in a fixed order, by mean_loss_block().
__global__ __launch_bounds__(TB) void k_softmax_xent(const float* __restrict__ Z, int64_t ld, int B, int C,
                                                     const int32_t* __restrict__ labels,
                                                     const int32_t* __restrict__ seeds, float* __restrict__ dZ,
                                                     float* __restrict__ row_loss) {
    const int lane = threadIdx.x & 63;
    const int row = (blockIdx.x * TB + threadIdx.x) >> 6;
    if (row >= B) return;
    const float* z = Z + (int64_t)row * ld;
    const int y = labels[seeds ? seeds[row] : row];
    float mx = -INFINITY;
    for (int c = lane; c < C; c += 64) mx = fmaxf(mx, z[c]);
    mx = wave_max(mx);
    float s = 0.f;
    for (int c = lane; c < C; c += 64) s += expf(z[c] - mx);
    s = wave_sum(s);
    const float invB = 1.0f / (float)B;
    for (int c = lane; c < C; c += 64) {
        const float p = expf(z[c] - mx) / s;
        dZ[(int64_t)row * C + c] = (p - (c == y ? 1.f : 0.f)) * invB;
    }
    if (lane == 0) row_loss[row] = logf(s) + mx - z[y];
}

}  // namespace

int32_t softmax_xent(const float* logits, int64_t ld, int32_t B, int32_t C, const int32_t* labels,
                     const int32_t* seeds, float* dZ, float* row_loss, hipStream_t st) {
    if (B <= 0) return SDT_OK;
    hipLaunchKernelGGL(k_softmax_xent, dim3(ceil_div(B, TB / WAVE)), dim3(TB), 0, st, logits, ld, B, C, labels, seeds,
                       dZ, row_loss);
    SDT_CHECK_LAUNCH("softmax_xent");
    return SDT_OK;
}

}  // namespace sdt

extern "C" const char* sdt_version(void) { return "0.1.0"; }
extern "C" const char* sdt_last_error(void) { return sdt::g_err; }
