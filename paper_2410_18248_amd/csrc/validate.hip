// A debug aid: checks the device-resident arguments of a decode call, which the calls
// themselves never validate (they make no host synchronisation).  Reads the block table, the
// context lengths and the running mask only; the K/V pools are not touched.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace lamps {
namespace {

// One workgroup per request.  result: [0] number of bad requests, [1] lowest bad request
// (initialised to INT_MAX by the launcher's fill), [2]/[3] reason and value for that request
// (written by whoever holds the lowest index after the count is final: a second, tiny pass).
__global__ __launch_bounds__(256) void validate_args(const int32_t *block_table, const int32_t *ctx_lens,
                                                     const uint8_t *running, int32_t max_blocks,
                                                     int32_t block_size, int32_t num_blocks, int32_t *bad)
{
    const int r = blockIdx.x;
    const int C = ctx_lens[r];
    __shared__ int first_bad_entry;
    if (threadIdx.x == 0) first_bad_entry = 0x7fffffff;
    __syncthreads();
    const long long cap = (long long)max_blocks * block_size;
    int reason = 0, value = 0;
    if (C < 0 || C > cap) {
        reason = 1;
        value = C;
    } else if (running[r]) {
        const int nb = (C + block_size - 1) / block_size;
        for (int j = threadIdx.x; j < nb; j += blockDim.x) {
            const int b = block_table[(size_t)r * max_blocks + j];
            if (b < 0 || b >= num_blocks) atomicMin(&first_bad_entry, j);
        }
        __syncthreads();
        if (first_bad_entry != 0x7fffffff) {
            reason = 2;
            value = block_table[(size_t)r * max_blocks + first_bad_entry];
        }
    }
    if (threadIdx.x == 0) {
        bad[4 + 2 * r] = reason;
        bad[4 + 2 * r + 1] = value;
    }
}

// Folds the per-request verdicts: count, lowest bad request, its reason and value.
__global__ __launch_bounds__(256) void validate_fold(int32_t batch, int32_t *bad)
{
    __shared__ int count, lowest;
    if (threadIdx.x == 0) {
        count = 0;
        lowest = 0x7fffffff;
    }
    __syncthreads();
    for (int r = threadIdx.x; r < batch; r += blockDim.x)
        if (bad[4 + 2 * r]) {
            atomicAdd(&count, 1);
            atomicMin(&lowest, r);
        }
    __syncthreads();
    if (threadIdx.x == 0) {
        bad[0] = count;
        bad[1] = count ? lowest : -1;
        bad[2] = count ? bad[4 + 2 * lowest] : 0;
        bad[3] = count ? bad[4 + 2 * lowest + 1] : 0;
    }
}

}  // namespace

hipError_t launch_validate(const int32_t *block_table, const int32_t *ctx_lens, const uint8_t *running,
                           int32_t batch, int32_t max_blocks, int32_t block_size, int32_t num_blocks,
                           int32_t *result, hipStream_t stream)
{
    if (batch <= 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(validate_args, dim3((unsigned)batch), dim3(256), 0, stream, block_table, ctx_lens, running,
                       max_blocks, block_size, num_blocks, result);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(validate_fold, dim3(1), dim3(256), 0, stream, batch, result);
    return hipGetLastError();
}

}  // namespace lamps
