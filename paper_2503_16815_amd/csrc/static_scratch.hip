// deft_knapsack_solve_batch_static: the sequential mode for callers that cannot
// allocate (code under HIP graph capture, serving loops, harnesses that forbid
// hipMalloc).  It has no handle.  Everything a handle would own - the keep table and
// the offered-item lists of the LDS-resident-row kernels - lives in one file-scope
// device array of a fixed, modest size; the kernels are the handle path's own and take
// the array's address as their scratch argument.
//
// The array exists once per GPU the library runs on, for the life of the process.  Its
// name is a host-side stand-in, not a device address: the address on each device comes
// from hipGetSymbolAddress, looked up once per device with that device current, and only
// that address is ever handed to a kernel.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>

#include "kernels.h"

using namespace deft;

namespace {

constexpr int64_t kStaticScratchBytes = DEFT_STATIC_SCRATCH_BYTES;
static_assert(kStaticScratchBytes % 256 == 0, "whole 256-byte lines");

static __device__ __attribute__((used)) __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
constexpr int kVariants = 8;  // entries of the LDS-row kernel table

struct PerDevice {
    bool ready = false;
    bool usable = false;       // a gfx950
    void *ptr = nullptr;       // this device's copy of `scratch`
    int lds_per_wg = 0;
    bool prepared[kVariants] = {};
};
PerDevice g_dev[kMaxDevices];
std::mutex g_mutex;

struct DeviceScope {
    int prev = -1;
    bool ok = false;
    explicit DeviceScope(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = (prev == dev) || hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceScope()
    {
        if (ok && prev >= 0) (void)hipSetDevice(prev);
    }
};

// First call on a device (that device current): architecture check, the address of this
// device's copy of the array.
deft_status_t device_setup(int device, PerDevice **out)
{
    PerDevice &d = g_dev[device];
    if (!d.ready) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, device) != hipSuccess) {
            (void)hipGetLastError();
            return DEFT_ERR_DEVICE;
        }
        d.usable = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0;
        d.lds_per_wg = (int)prop.sharedMemPerBlockOptin > 0 ? (int)prop.sharedMemPerBlockOptin
                                                            : (int)prop.sharedMemPerBlock;
        if (d.usable) {
            void *p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
                (void)hipGetLastError();
                return DEFT_ERR_DEVICE;
            }
            d.ptr = p;
        }
        d.ready = true;
    }
    *out = &d;
    return d.usable ? DEFT_OK : DEFT_ERR_DEVICE;
}

}  // namespace

extern "C" deft_status_t deft_knapsack_solve_batch_static(int32_t device, int32_t max_capacity,
                                                          const deft_knapsack_batch_t *b)
{
    if (!b || device < 0 || max_capacity < 1) return DEFT_ERR_INVALID_ARG;
    if (b->mode != DEFT_MODE_SEQUENTIAL) return DEFT_ERR_INVALID_ARG;
    if (b->batch < 0 || b->item_stride < 1 || b->knap_stride < 1) return DEFT_ERR_INVALID_ARG;
    if (!b->n_items || !b->n_knapsacks || !b->weights || !b->values || !b->capacities || !b->total_value ||
        !b->knap_value || !b->knap_load || !b->assignment || !b->status)
        return DEFT_ERR_INVALID_ARG;
    if (device >= kMaxDevices || b->item_stride > 4096 || b->knap_stride > 64) return DEFT_ERR_LIMIT;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess) {
        (void)hipGetLastError();
        return DEFT_ERR_DEVICE;
    }
    if (device >= ndev) return DEFT_ERR_INVALID_ARG;
    if (b->batch == 0) return DEFT_OK;

    DeviceScope scope(device);
    if (!scope.ok) return DEFT_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_mutex);
    PerDevice *d = nullptr;
    const deft_status_t rc = device_setup(device, &d);
    if (rc != DEFT_OK) return rc;

    // the same plan a handle with these limits would get; rows that need global memory,
    // and batches whose keep table and lists exceed the array, are refused
    SeqLdsPlan plan{};
    if (!seq_lds_plan(max_capacity, b->item_stride, b->knap_stride, b->batch, d->lds_per_wg, false, &plan))
        return DEFT_ERR_LIMIT;
    if (plan.scratch_bytes > kStaticScratchBytes) return DEFT_ERR_LIMIT;
    if (plan.variant < 0 || plan.variant >= kVariants) return DEFT_ERR_DEVICE;
    if (!d->prepared[plan.variant]) {  // once per device and kernel: the dynamic-LDS attribute
        if (seq_lds_prepare(&plan) != hipSuccess) {
            (void)hipGetLastError();
            return DEFT_ERR_DEVICE;
        }
        d->prepared[plan.variant] = true;
    }

    BatchArgs a{};
    a.mode = DEFT_MODE_SEQUENTIAL;
    a.batch = b->batch;
    a.item_stride = b->item_stride;
    a.knap_stride = b->knap_stride;
    a.max_capacity = max_capacity;
    a.n_items = b->n_items;
    a.n_knapsacks = b->n_knapsacks;
    a.weights = b->weights;
    a.values = b->values;
    a.capacities = b->capacities;
    a.fill_order = b->fill_order;
    a.drop_time = nullptr;
    a.total_value = b->total_value;
    a.knap_value = b->knap_value;
    a.knap_load = b->knap_load;
    a.assignment = b->assignment;
    a.status = b->status;
    // Nothing in the array has to start at zero: a stage writes its item list before any
    // lane reads it, and a keep-row part is read only when the flag its writer set in
    // registers says it was written in this launch.  What the last call left is never read.
    if (seq_lds_launch(plan, a, d->ptr, static_cast<hipStream_t>(b->stream), nullptr) != hipSuccess) {
        (void)hipGetLastError();
        return DEFT_ERR_DEVICE;
    }
    return DEFT_OK;
}
