// pxr_render_batch_kinematic_static: joint angles in, frames out, for callers that cannot allocate device
// memory or hand over a workspace (code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc).  The poses that pass from the kinematics kernel to the render kernel live in a file-scope
// device array instead of a caller-provided buffer.  Each GPU the library runs on holds its own copy of the
// array, at its own address, until the process ends.

#include <hip/hip_runtime.h>

#include <mutex>

#include "pxr_internal.h"

namespace {

// B * S * n_bodies * 28 bytes of poses must fit.  32 MiB = 79 891 frames of a 15-body scene (16 384 environments
// x 3 steps of the humanoid-and-box scene need 20.6 MB).
constexpr size_t kScratchBytes = 32u << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// In host code the array's name is a stand-in, not a device address: the address is looked up once per device,
// with that device current, and only the looked-up pointer is ever handed to a kernel.
constexpr int kMaxDevices = 64;
std::mutex g_mu;
float* g_ptr[kMaxDevices] = {};

}  // namespace

int pxr::static_pose_scratch(float** out, size_t* capacity_bytes, std::string& err) {
    int device = -1;
    hipError_t rc = hipGetDevice(&device);
    if (rc != hipSuccess || device < 0 || device >= kMaxDevices) {
        err = rc != hipSuccess ? std::string("hipGetDevice failed: ") + hipGetErrorString(rc)
                               : "device index beyond the 64 this table holds";
        return PXR_ERR_DEVICE;
    }
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_ptr[device]) {
        void* p = nullptr;
        rc = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (rc != hipSuccess || !p) {
            err = std::string("hipGetSymbolAddress(scratch) failed: ") + hipGetErrorString(rc);
            return PXR_ERR_DEVICE;
        }
        g_ptr[device] = static_cast<float*>(p);
    }
    *out = g_ptr[device];
    if (capacity_bytes) *capacity_bytes = kScratchBytes;
    return PXR_OK;
}
