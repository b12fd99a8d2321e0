// Mean loss at a given theta for callers that cannot allocate device memory: the partial sums of the loss kernel go to
// a file-scope device array instead of a context's workspace, and the result is left in device memory, so the call
// enqueues two kernels and nothing else (no allocation, no copy, no synchronisation).
#include "../../include/bmgd.h"
#include "bmgd_internal.h"

#include <stdio.h>

#include <algorithm>
#include <mutex>

using namespace bmgd;

namespace {

// One partial sum per workgroup of the loss kernel: kEvalBlocks doubles = 8 KiB on every device the library runs on,
// held until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the address the
// kernels are given is looked up once per device (g_scratch) and nothing else in host code uses the name.
static __device__ __align__(256) double scratch[kEvalBlocks];

constexpr int kMaxDevices = 64;
double* g_scratch[kMaxDevices];                  // device address of `scratch` on device d, NULL until looked up
std::mutex g_scratch_mu;

// Adds the partial sums in index order (the order the host uses in bmgd_eval_loss) and divides by the row count.
__global__ void __launch_bounds__(256) mean_of_partials_kernel(const double* __restrict__ partial, int n, double rows,
                                                               double* __restrict__ out)
{
    __shared__ double part[kEvalBlocks];
    for (int i = threadIdx.x; i < n; i += 256) part[i] = partial[i];
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int i = 0; i < n; ++i) t += part[i];
        *out = t / rows;
    }
}

int fail_static(int code, const char* msg)
{
    set_create_error(msg);
    return code;
}

int hip_fail_static(hipError_t e, const char* what)
{
    char buf[256];
    snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(e));
    (void)hipGetLastError();
    return fail_static(BMGD_EHIP, buf);
}

}  // namespace

extern "C" __attribute__((visibility("default")))
int bmgd_eval_loss_static(int32_t model, const float* dev_x, const float* dev_y, const float* dev_theta, int64_t rows,
                          int64_t p, void* stream, double* dev_out)
{
    if (model == BMGD_SOFTMAX)
        return fail_static(BMGD_EINVAL, "bmgd_eval_loss_static: softmax needs a logits scratch of rows x classes floats, "
                                        "beyond the 8 KiB static array; use bmgd_eval_loss");
    if (model != BMGD_LINEAR && model != BMGD_LOGISTIC) return fail_static(BMGD_EINVAL, "bmgd_eval_loss_static: unknown model");
    if (!dev_x || !dev_y || !dev_theta || !dev_out)
        return fail_static(BMGD_EINVAL, "bmgd_eval_loss_static: dev_x, dev_y, dev_theta and dev_out must not be NULL");
    if (p < 1 || p > 4096) return fail_static(BMGD_EINVAL, "bmgd_eval_loss_static: p must be in [1, 4096]");
    if (rows < 1 || rows >= (int64_t(1) << 30)) return fail_static(BMGD_EINVAL, "bmgd_eval_loss_static: rows must be in [1, 2^30)");
    if ((reinterpret_cast<uintptr_t>(dev_x) % 16) != 0 || (reinterpret_cast<uintptr_t>(dev_y) % 4) != 0 ||
        (reinterpret_cast<uintptr_t>(dev_theta) % 4) != 0 || (reinterpret_cast<uintptr_t>(dev_out) % 8) != 0)
        return fail_static(BMGD_EINVAL, "bmgd_eval_loss_static: dev_x must be 16-byte, dev_out 8-byte, the others 4-byte aligned");
    const int nblocks = (int)std::min<int64_t>(kEvalBlocks, (rows + 3) / 4);     // never more partial sums than the array holds

    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail_static(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail_static(BMGD_EINVAL, "bmgd_eval_loss_static: device index above 63");
    double* part = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mu);
        if (!g_scratch[dev]) {
            // each device holds its own copy of the array at its own address
            void* addr = nullptr;
            e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !addr) return hip_fail_static(e, "hipGetSymbolAddress(scratch)");
            g_scratch[dev] = static_cast<double*>(addr);
        }
        part = g_scratch[dev];
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    e = glm_launch_loss(dev_x, dev_y, dev_theta, (int)rows, (int)p, model, part, nblocks, s);
    if (e != hipSuccess) return hip_fail_static(e, "launch of the loss kernel");
    hipLaunchKernelGGL(mean_of_partials_kernel, dim3(1), dim3(256), 0, s, part, nblocks, (double)rows, dev_out);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail_static(e, "launch of the final sum");
    return BMGD_OK;
}
