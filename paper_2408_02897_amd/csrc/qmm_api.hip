// Small host-only entry points of the C ABI.
#include <atomic>
#include "qmm_device.h"

// The ring of arrival counters of the single-launch reductions (qmm_device.h): part of the device image, so zero
// when the image is loaded; every kernel that uses a slot leaves it zero.  `arrival_ring` is the host-side stand-in
// of the device array: its address on a GPU is looked up once per device and only that address goes to kernels.
static __device__ __align__(256) uint32_t arrival_ring[qmm::kArrivalSlots * qmm::kArrivalWords];
namespace qmm {
namespace {
constexpr int kMaxDevices = 64;
std::atomic<uint32_t*> ring_addr[kMaxDevices];
std::atomic<uint32_t> next_slot{0};
}  // namespace
qmm_status arrival_slots(int count, uint32_t** first)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return QMM_ERR_LAUNCH;
    if (dev < 0 || dev >= kMaxDevices || count < 1 || count > 8) return QMM_ERR_UNSUPPORTED;
    uint32_t* p = ring_addr[dev].load(std::memory_order_acquire);
    if (!p) {
        void* q = nullptr;
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(arrival_ring)) != hipSuccess || !q) return QMM_ERR_LAUNCH;
        p = static_cast<uint32_t*>(q);
        ring_addr[dev].store(p, std::memory_order_release);
    }
    // slots are taken in aligned groups of eight so that a call's `count` slots never wrap around the ring
    const uint32_t group = next_slot.fetch_add(1, std::memory_order_relaxed) % (kArrivalSlots / 8);
    *first = p + (size_t)group * 8 * kArrivalWords;
    return QMM_OK;
}
}  // namespace qmm

extern "C" const char* qmm_status_string(qmm_status s)
{
    switch (s) {
    case QMM_OK: return "ok";
    case QMM_ERR_NULL: return "required pointer is NULL";
    case QMM_ERR_SHAPE: return "invalid shape or stride";
    case QMM_ERR_ENUM: return "invalid enum value";
    case QMM_ERR_ALIGN: return "alignment rule violated";
    case QMM_ERR_UNSUPPORTED: return "not supported by this build";
    case QMM_ERR_WORKSPACE: return "workspace missing or too small";
    case QMM_ERR_LAUNCH: return "kernel launch failed";
    case QMM_ERR_LIMIT: return "input exceeds a fixed capacity of the call";
    }
    return "unknown status";
}

extern "C" int qmm_version(void) { return 100; }
