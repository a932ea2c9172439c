// Cache maintenance of a compressed layer (paper section 3.2.1: only sink and recent
// tokens are kept): append one token per sequence into the page its logical page owns.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace omniattn {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// One work group per sequence; thread t copies 16 bytes of the new row.
__global__ __launch_bounds__(128) void append_kernel(AppendParams p) {
  const int b = blockIdx.x;
  const int L = p.seq_lens[b];
  const int lp = L / kPage;
  if (L < 0 || lp >= p.max_pages) return;  // full (or invalid): leave the sequence alone
  const int phys = p.seq_pages[(size_t)b * p.ring_pages + ring_slot(p.S, p.W, lp)];
  const int slot = L - lp * kPage;
  const int t = threadIdx.x;
  if (t * 16 < p.row_bytes)
    *(u32x4*)(p.kv + ((size_t)phys * kPage + slot) * p.row_bytes + t * 16) =
        *(const u32x4*)(p.new_rows + (size_t)b * p.row_bytes + t * 16);
  __syncthreads();  // every thread has read L before it changes
  if (t == 0) {
    if (p.new_scales) p.kv_scales[(size_t)phys * kPage + slot] = p.new_scales[b];
    if (slot == 0) p.page_table[(size_t)b * p.max_pages + lp] = phys;
    p.seq_lens[b] = L + 1;
  }
}

hipError_t launch_append(const AppendParams& p, int batch, hipStream_t stream) {
  if (batch <= 0) return hipSuccess;
  hipLaunchKernelGGL(append_kernel, dim3(batch), dim3(128), 0, stream, p);
  return hipGetLastError();
}

}  // namespace omniattn
