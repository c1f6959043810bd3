// Batched gather-pack (HBM -> pinned host staging) and scatter-unpack (staging -> HBM)
// copy kernels for gfx950.
//
// Swap-out moves a tensor to host memory after its last forward use, swap-in
// brings it back before its first backward use (Sec. 1, Sec. 5.2 of the
// SmartSwap paper).  The paper issues one framework copy per tensor; small
// tensors then waste the link (Sec. 4.2).  Here one launch moves a whole batch
// of variable-size tensors: the batch is cut into chunks (64 KiB, smaller for a
// small batch so that every workgroup of the grid has work), a small
// persistent grid walks the chunks, and each workgroup looks its chunk's
// descriptor up in a per-chunk table built when the schedule is loaded (two
// dependent loads per chunk, no search, no LDS).  All
// traffic is 16 bytes per lane, a wavefront touching 1 KiB of consecutive
// addresses on both sides; a byte tail handles sizes that are not multiples of
// 16.  The staging area is host memory mapped into the device address space,
// so the stores (swap-out) or loads (swap-in) cross the host link directly.
//
// The path is bound by the host link (tens of GB/s), not by HBM (8 TB/s): a few
// dozen workgroups saturate it, which leaves the compute units to the
// training step running on the compute stream.
#include "ss_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// kUnroll 16-byte accesses are in flight per lane before the first store is issued.
template <bool TO_HOST, uint32_t kUnroll>
__global__ __launch_bounds__(SS_COPY_THREADS) void ss_copy_kernel(
    uint8_t *__restrict__ arena, uint8_t *__restrict__ staging, const ss_desc_t *__restrict__ descs,
    const uint32_t *__restrict__ chunk0, const uint32_t *__restrict__ chunk_desc, uint32_t n_chunks,
    uint32_t chunk_shift) {
  const uint32_t chunk_bytes = 1u << chunk_shift;     // 4 KiB .. 64 KiB, chosen per batch
  const uint32_t tid = threadIdx.x;
  for (uint32_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    // chunk_desc[c]: the descriptor chunk c belongs to; chunk0[d]: first chunk of descriptor d
    const uint32_t lo = chunk_desc[c];
    const ss_desc_t d = descs[lo];
    const uint64_t off = (uint64_t)(c - chunk0[lo]) << chunk_shift;
    const uint64_t left = d.nbytes - off;
    const uint32_t n = left < chunk_bytes ? (uint32_t)left : chunk_bytes;
    const uint8_t *src = TO_HOST ? arena + d.dev_off + off : staging + d.host_off + off;
    uint8_t *dst = TO_HOST ? staging + d.host_off + off : arena + d.dev_off + off;

    const u32x4 *src16 = reinterpret_cast<const u32x4 *>(src);
    u32x4 *dst16 = reinterpret_cast<u32x4 *>(dst);
    const uint32_t n16 = n >> 4;
    for (uint32_t base = 0; base < n16; base += SS_COPY_THREADS * kUnroll) {
      u32x4 v[kUnroll];
#pragma unroll
      for (uint32_t u = 0; u < kUnroll; ++u) {
        const uint32_t i = base + u * SS_COPY_THREADS + tid;
        if (i < n16) v[u] = __builtin_nontemporal_load(src16 + i);
      }
#pragma unroll
      for (uint32_t u = 0; u < kUnroll; ++u) {
        const uint32_t i = base + u * SS_COPY_THREADS + tid;
        if (i < n16) __builtin_nontemporal_store(v[u], dst16 + i);
      }
    }
    const uint32_t tail = n & 15u;          // only the last chunk of a tensor can have one
    if (tid < tail) dst[(n16 << 4) + tid] = src[(n16 << 4) + tid];
  }
}

__global__ __launch_bounds__(256) void ss_fill_kernel(uint8_t *dst, uint64_t nbytes, uint32_t word) {
  // dst is 16-byte aligned (checked by the caller)
  const uint64_t n16 = nbytes >> 4;
  u32x4 w = {word, word, word, word};
  u32x4 *d16 = reinterpret_cast<u32x4 *>(dst);
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
       i += (uint64_t)gridDim.x * blockDim.x)
    d16[i] = w;
  if (blockIdx.x == 0 && threadIdx.x < (nbytes & 15u)) dst[(n16 << 4) + threadIdx.x] = (uint8_t)word;
}

}  // namespace

void ss_launch_copy(hipStream_t s, uint32_t workgroups, uint32_t unroll, bool to_host, uint8_t *arena,
                    uint8_t *staging, const ss_desc_t *d_descs, const uint32_t *d_chunk0,
                    const uint32_t *d_chunk_desc, uint32_t n_chunks, uint32_t chunk_shift) {
  if (n_chunks == 0) return;
  const dim3 grid(workgroups < n_chunks ? workgroups : n_chunks), block(SS_COPY_THREADS);
#define SS_LAUNCH(TH, U)                                                                                  \
  hipLaunchKernelGGL((ss_copy_kernel<TH, U>), grid, block, 0, s, arena, staging, d_descs, d_chunk0,        \
                     d_chunk_desc, n_chunks, chunk_shift)
  if (to_host) {
    if (unroll <= 2) SS_LAUNCH(true, 2); else if (unroll <= 4) SS_LAUNCH(true, 4); else SS_LAUNCH(true, 8);
  } else {
    if (unroll <= 2) SS_LAUNCH(false, 2); else if (unroll <= 4) SS_LAUNCH(false, 4); else SS_LAUNCH(false, 8);
  }
#undef SS_LAUNCH
}

void ss_launch_fill(hipStream_t s, uint8_t *dst, uint64_t nbytes, uint8_t value) {
  if (nbytes == 0) return;
  uint32_t word = value * 0x01010101u;
  uint64_t n16 = nbytes >> 4;
  uint32_t grid = (uint32_t)((n16 + 255) / 256);
  if (grid == 0) grid = 1;
  if (grid > 1024) grid = 1024;
  hipLaunchKernelGGL(ss_fill_kernel, dim3(grid), dim3(256), 0, s, dst, nbytes, word);
}
