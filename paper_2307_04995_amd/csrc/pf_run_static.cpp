// pf_chain_run_static: plan and run a chain without allocating anything on the device.
//
// Whatever device memory the chain's kernels need beyond its inputs and outputs (per-workgroup partial statistics
// of a GroupNorm, per-slice partial results and arrival counters of the one-token attention) is taken from one
// file-scope device array of fixed size instead of hipMalloc.  Every device the library runs on holds its own
// copy of that array until the process ends; its address on a device is looked up once, with that device
// current, and kept.  All calls on a device share the array: it keeps the previous call's contents, so the parts
// that must start at a value are rewritten by a small fill kernel on the caller's stream before the chain's
// kernels, and two calls that overlap in time on one device race.
#include <mutex>

#include "pf_host_internal.h"

using namespace pfh;

namespace {

typedef uint32_t pf_uint4_t __attribute__((ext_vector_type(4)));

constexpr uint64_t kScratchBytes = PF_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device ordinal; null until looked up

// The address of the array on `device`, which must be the current device.
pf_status scratch_on_device(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) return fail(PF_ERR_INVALID_ARG, "device ordinal %d out of range", device);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return fail(PF_ERR_HIP, "cannot locate the static scratch array on device %d: %s", device, hipGetErrorString(e));
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return PF_OK;
}

// n 16-byte vectors at p := the byte pattern repeated (a fill kernel, not a memset node: the launch may be recorded
// into a graph by the caller)
__global__ void __launch_bounds__(256) fill_scratch_kernel(pf_uint4_t* p, uint32_t word, uint64_t n) {
    const uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (i < n) p[i] = pf_uint4_t{word, word, word, word};
}

struct DeviceRestore {
    int prev = -1;
    ~DeviceRestore() {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

}  // namespace

extern "C" pf_status pf_chain_run_static(const pf_chain_desc* desc, int32_t device, const void* const* inputs, void* const* outputs, void* stream) {
    if (!desc || !inputs || !outputs) return fail(PF_ERR_INVALID_ARG, "null argument");
    DeviceRestore restore;
    if (hipGetDevice(&restore.prev) != hipSuccess) restore.prev = -1;
    if (hipSetDevice(device) != hipSuccess) return fail(PF_ERR_HIP, "cannot select device %d", device);
    void* base = nullptr;
    pf_status s = scratch_on_device(device, &base);
    if (s != PF_OK) return s;

    ScratchArena arena{static_cast<char*>(base), kScratchBytes, 0};
    pf_plan* plan = nullptr;
    tls_scratch = &arena;
    s = plan_one_kernel(desc, device, -1, &plan);
    tls_scratch = nullptr;
    if (s != PF_OK) return s;

    hipStream_t st = (hipStream_t)stream;
    for (const pf_plan_s::Fill& f : plan->fills) {
        // regions are carved at 256-byte boundaries and sized in whole 16-byte vectors by the planner
        const uintptr_t off = (uintptr_t)((char*)f.ptr - (char*)base);
        if (off % 16 != 0 || f.bytes % 16 != 0 || off + f.bytes > kScratchBytes) {
            pf_chain_plan_destroy(plan);
            return fail(PF_ERR_INVALID_ARG, "internal: scratch region out of bounds");
        }
        const uint64_t n = f.bytes / 16;
        const uint32_t b = (uint32_t)(f.byte & 0xff);
        hipLaunchKernelGGL(fill_scratch_kernel, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0, st, reinterpret_cast<pf_uint4_t*>(f.ptr),
                           b * 0x01010101u, n);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            pf_chain_plan_destroy(plan);
            return fail(PF_ERR_HIP, "fill kernel launch failed: %s", hipGetErrorString(e));
        }
    }
    s = pf_chain_run(plan, inputs, outputs, stream);
    pf_chain_plan_destroy(plan);  // kernel arguments were copied at launch; the scratch array is not the plan's to free
    return s;
}
