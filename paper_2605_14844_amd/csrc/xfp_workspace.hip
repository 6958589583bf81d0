// The static ring of workspaces: device memory the entry points use beyond their
// inputs and outputs (re-laid activations of the batched kernel, fp32 planes for
// split-K partial sums and for unfused epilogues).  Nothing is ever allocated:
// the ring is a file-scope device array, every GPU of the process holds its own
// copy, and a call that needs scratch takes ONE slot, whatever it needs of it.
#include "xfp_internal.h"

#include <atomic>

namespace xfp {

namespace {

// Eager calls cycle through the first kEagerSlots slots.  A call recorded into a
// HIP graph keeps its slot for as long as the graph lives, so recorded calls
// cycle through kCaptureSlots slots of their own: a graph replayed on one stream
// never meets an eager call on another in the same slot.
constexpr int kEagerSlots = 4;
constexpr int kCaptureSlots = 4;
static_assert(sizeof(WorkspaceLayout) % 256 == 0, "slots stay 256-byte aligned");
__device__ __align__(256) unsigned char g_ring[kEagerSlots + kCaptureSlots][sizeof(WorkspaceLayout)];

std::atomic<void *> g_ring_base[kMaxDevices];      // device address of g_ring, per device
std::atomic<unsigned> g_ticket_eager{0}, g_ticket_capture{0};

}  // namespace

int ring_slots(bool capturing) { return capturing ? kCaptureSlots : kEagerSlots; }

int ring_slot_index(unsigned ticket, bool capturing)
{
    return capturing ? kEagerSlots + (int)(ticket % kCaptureSlots) : (int)(ticket % kEagerSlots);
}

hipError_t ring_resolve()
{
    const int dev = current_device();
    if (dev < 0) return hipErrorInvalidDevice;
    if (g_ring_base[dev].load(std::memory_order_acquire)) return hipSuccess;
    void *p = nullptr;
    hipError_t err = hipGetSymbolAddress(&p, HIP_SYMBOL(g_ring));
    if (err != hipSuccess) return err;
    g_ring_base[dev].store(p, std::memory_order_release);
    return hipSuccess;
}

hipError_t ring_workspace(hipStream_t s, Workspace *out)
{
    hipError_t err = ring_resolve();
    if (err != hipSuccess) return err;
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    err = hipStreamIsCapturing(s, &st);
    if (err != hipSuccess) return err;
    const bool capturing = st != hipStreamCaptureStatusNone;
    const unsigned ticket = (capturing ? g_ticket_capture : g_ticket_eager).fetch_add(1, std::memory_order_relaxed);
    unsigned char *base = static_cast<unsigned char *>(g_ring_base[current_device()].load(std::memory_order_acquire));
    *out = workspace_at(base + (size_t)ring_slot_index(ticket, capturing) * sizeof(WorkspaceLayout));
    return hipSuccess;
}

}  // namespace xfp
