// Device -> pinned-host copies on the DMA engines (see dma_copy.cpp).
#pragma once
#include <cstddef>
#include <new>

namespace pmx {
struct DmaCopy;
// Looks up the agents that own the two example pointers (a hipMalloc and a hipHostMalloc allocation of the
// stage's device).  Returns nullptr if the HSA runtime refuses anything: the caller then keeps using the
// runtime's own copies.
DmaCopy* dma_copy_create(const void* a_device_pointer, const void* a_pinned_host_pointer);
void dma_copy_destroy(DmaCopy* d);
// Blocks until the copy has completed.  0 = done, negative = the copy was refused or did not finish in 10 s.
int dma_copy_d2h(DmaCopy* d, void* dst_host, const void* src_dev, size_t bytes);
}  // namespace pmx
