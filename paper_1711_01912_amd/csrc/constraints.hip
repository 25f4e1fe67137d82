// Validity of candidate partitions under the placement constraints of the problem
// statement (paper, section 2): collocation pairs must share a device, device
// constraints fix a vertex's device.  One workgroup per partition; its threads take
// the constraints in turn and count the broken ones.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "cpeval_internal.hpp"
#include "launch.hpp"

namespace cpeval {

namespace {

__global__ __launch_bounds__(256) void validate_kernel(const uint8_t *__restrict__ assign, int64_t a_stride_p,
                                                       int64_t a_stride_v, int32_t n, int32_t P, int32_t k,
                                                       int64_t num_pairs, const int32_t *__restrict__ pairs,
                                                       int64_t num_pins, const int32_t *__restrict__ pins,
                                                       uint8_t *__restrict__ valid, int32_t *__restrict__ violations,
                                                       int32_t *status) {
    __shared__ int32_t wave_sum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    bool bad_index = false;
    for (int32_t q = blockIdx.x; q < P; q += gridDim.x) {
        const uint8_t *row = assign + (int64_t)q * a_stride_p;
        int32_t broken = 0;
        for (int64_t i = tid; i < num_pairs; i += 256) {
            const int32_t u = pairs[2 * i], v = pairs[2 * i + 1];
            if ((uint32_t)u >= (uint32_t)n || (uint32_t)v >= (uint32_t)n) { bad_index = true; continue; }
            broken += row[(int64_t)u * a_stride_v] != row[(int64_t)v * a_stride_v];
        }
        for (int64_t i = tid; i < num_pins; i += 256) {
            const int32_t v = pins[2 * i], d = pins[2 * i + 1];
            if ((uint32_t)v >= (uint32_t)n || (uint32_t)d >= (uint32_t)k) { bad_index = true; continue; }
            broken += (int32_t)row[(int64_t)v * a_stride_v] != d;
        }
        for (int off = 32; off > 0; off >>= 1) broken += __shfl_xor(broken, off);
        if (lane == 0) wave_sum[wave] = broken;
        __syncthreads();
        if (tid == 0) {
            const int32_t total = wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
            valid[q] = total == 0;
            if (violations) violations[q] = total;
        }
        __syncthreads();
    }
    if (bad_index) atomicOr(status, CP_STATUS_BAD_CONSTRAINT);
}

}  // namespace

int launch_validate(const uint8_t *assign, int64_t a_stride_p, int64_t a_stride_v, int32_t n, int32_t P, int32_t k,
                    int64_t num_pairs, const int32_t *pairs, int64_t num_pins, const int32_t *pins,
                    uint8_t *valid, int32_t *violations, int32_t *status, void *stream) {
    const unsigned blocks = (unsigned)std::min<int32_t>(P, 256 * 8);
    hipLaunchKernelGGL(validate_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, assign, a_stride_p,
                       a_stride_v, n, P, k, num_pairs, pairs, num_pins, pins, valid, violations, status);
    return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_HIP;
}

}  // namespace cpeval
