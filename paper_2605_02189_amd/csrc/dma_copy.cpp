// Device -> pinned-host copies on the GPU's DMA engines, through the HSA runtime that HIP itself sits on.
//
// Why not hipMemcpyAsync: this runtime executes a device-to-host hipMemcpyAsync as a shader copy with a
// full-size grid, and a kernel that runs beside it takes several times longer for the duration of the copy
// (measured on the KV write-back of a prefill pass: a 130 us attention launch took 660 us next to a 33 MB copy).
// hsa_amd_memory_async_copy uses an SDMA engine, as the host-to-device prefetch copies already do.
//
// Only the write-back worker thread calls copy(); it blocks until the copy has completed.
#include <hsa/hsa.h>
#include <hsa/hsa_ext_amd.h>

#include <cstdint>
#include <cstdlib>

#include "dma_copy.hpp"

namespace pmx {

struct DmaCopy {
  hsa_agent_t gpu{}, cpu{};
  hsa_signal_t sig{};
  bool have_sig = false;
};

namespace {
bool owner_of(const void* p, hsa_agent_t* out) {
  hsa_amd_pointer_info_t info{};
  info.size = sizeof(info);
  if (hsa_amd_pointer_info(const_cast<void*>(p), &info, nullptr, nullptr, nullptr) != HSA_STATUS_SUCCESS) return false;
  if (info.type == HSA_EXT_POINTER_TYPE_UNKNOWN) return false;
  *out = info.agentOwner;
  return true;
}
}  // namespace

DmaCopy* dma_copy_create(const void* a_device_pointer, const void* a_pinned_host_pointer) {
  if (getenv("PIPEMAX_NO_DMA_WRITEBACK")) return nullptr;      // tuning switch: the runtime's own copy instead
  if (hsa_init() != HSA_STATUS_SUCCESS) return nullptr;        // reference-counted; HIP has initialised it already
  DmaCopy* d = new (std::nothrow) DmaCopy();
  if (!d) { (void)hsa_shut_down(); return nullptr; }
  hsa_device_type_t tg{}, tc{};
  if (!owner_of(a_device_pointer, &d->gpu) || !owner_of(a_pinned_host_pointer, &d->cpu) ||
      hsa_agent_get_info(d->gpu, HSA_AGENT_INFO_DEVICE, &tg) != HSA_STATUS_SUCCESS || tg != HSA_DEVICE_TYPE_GPU ||
      hsa_agent_get_info(d->cpu, HSA_AGENT_INFO_DEVICE, &tc) != HSA_STATUS_SUCCESS || tc != HSA_DEVICE_TYPE_CPU ||
      hsa_signal_create(1, 0, nullptr, &d->sig) != HSA_STATUS_SUCCESS) {
    delete d;
    (void)hsa_shut_down();
    return nullptr;
  }
  d->have_sig = true;
  return d;
}

void dma_copy_destroy(DmaCopy* d) {
  if (!d) return;
  if (d->have_sig) (void)hsa_signal_destroy(d->sig);
  delete d;
  (void)hsa_shut_down();
}

int dma_copy_d2h(DmaCopy* d, void* dst_host, const void* src_dev, size_t bytes) {
  if (bytes == 0) return 0;
  hsa_signal_store_relaxed(d->sig, 1);
  if (hsa_amd_memory_async_copy(dst_host, d->cpu, src_dev, d->gpu, bytes, 0, nullptr, d->sig) != HSA_STATUS_SUCCESS)
    return -1;
  // blocked wait in slices of 100 ms, 10 s in all: a copy of a few tens of MB takes under a millisecond
  for (int i = 0; i < 100; ++i) {
    if (hsa_signal_wait_scacquire(d->sig, HSA_SIGNAL_CONDITION_LT, 1, 100ull * 1000 * 1000, HSA_WAIT_STATE_BLOCKED) < 1)
      return 0;
  }
  return -2;
}

}  // namespace pmx
