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
// dependent loads per chunk, no search, no LDS), and the loads of one block are
// issued before the stores of the block before it (software pipelining).  A
// second form of the kernel keeps the batch's chunk-prefix table in LDS and
// searches it per chunk instead (copy_desc_lookup = 1): it exists so that the
// two can be measured against each other; the per-chunk table is the default
// because it is faster on small tensors and never slower.  All
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

// One block of a chunk: at most SS_COPY_THREADS * kUnroll 16-byte vectors, plus (last block of a
// tensor only) a tail of fewer than 16 bytes.
struct CopyBlock {
  const u32x4 *src;
  u32x4 *dst;
  uint32_t n16;      // vectors in this block
  uint32_t tail;     // bytes after them (0..15)
};

// Walks the blocks one workgroup is responsible for: chunks blockIdx.x, blockIdx.x + gridDim.x, ...,
// each chunk cut into blocks of SS_COPY_THREADS * kUnroll vectors.
constexpr uint32_t kLdsPrefixMax = 8192;       // entries of the chunk-prefix table an LDS-lookup launch can hold (32 KiB)

template <bool TO_HOST, uint32_t kUnroll, bool LDS_LOOKUP>
struct BlockWalk {
  uint8_t *arena, *staging;
  const ss_desc_t *descs;
  const uint32_t *chunk0, *chunk_desc;
  const uint32_t *lds_prefix;   // LDS_LOOKUP: chunk0[0 .. n_desc] staged in LDS
  uint32_t n_desc;
  uint32_t n_chunks, chunk_shift;
  uint32_t c;          // current chunk
  uint32_t done16;     // vectors of the current chunk already handed out
  uint32_t left16;     // vectors of the current chunk still to hand out
  uint32_t tail;       // byte tail of the current chunk
  const uint8_t *src;
  uint8_t *dst;

  __device__ bool open_chunk() {
    if (c >= n_chunks) return false;
    // chunk_desc[c]: the descriptor chunk c belongs to; chunk0[d]: first chunk of descriptor d
    uint32_t lo, first;
    if (LDS_LOOKUP) {
      // the last descriptor whose first chunk is <= c (descriptors without bytes share their successor's
      // first chunk and are skipped by taking the last)
      uint32_t a = 0, b = n_desc;                 // invariant: prefix[a] <= c < prefix[b]
      while (b - a > 1) {
        const uint32_t m = (a + b) >> 1;
        if (lds_prefix[m] <= c) a = m; else b = m;
      }
      lo = a;
      first = lds_prefix[a];
    } else {
      lo = chunk_desc[c];
      first = chunk0[lo];
    }
    const ss_desc_t d = descs[lo];
    const uint64_t off = (uint64_t)(c - first) << chunk_shift;
    const uint64_t left = d.nbytes - off;
    const uint32_t n = left < (1ull << chunk_shift) ? (uint32_t)left : (1u << chunk_shift);
    src = TO_HOST ? arena + d.dev_off + off : staging + d.host_off + off;
    dst = TO_HOST ? staging + d.host_off + off : arena + d.dev_off + off;
    done16 = 0;
    left16 = n >> 4;
    tail = n & 15u;          // only the last chunk of a tensor can have one
    return true;
  }
  // next block, or false when this workgroup has no more; a chunk of fewer than 16 bytes yields one
  // block without vectors
  __device__ bool next(CopyBlock &b) {
    while (left16 == 0 && tail == 0) {
      c += gridDim.x;
      if (!open_chunk()) return false;
    }
    const uint32_t take = left16 < SS_COPY_THREADS * kUnroll ? left16 : SS_COPY_THREADS * kUnroll;
    b.src = reinterpret_cast<const u32x4 *>(src) + done16;
    b.dst = reinterpret_cast<u32x4 *>(dst) + done16;
    b.n16 = take;
    done16 += take;
    left16 -= take;
    b.tail = left16 == 0 ? tail : 0;
    if (left16 == 0) tail = 0;
    return true;
  }
};

// Software-pipelined: the kUnroll loads per lane of the next block are issued before the stores of the
// current one, so that each lane keeps requests on the host link in flight all the time (the link is a
// long pipe: what saturates it is bytes in flight, and with this a dozen workgroups hold as many as
// sixty-four did when loads and stores took turns).
template <bool TO_HOST, uint32_t kUnroll, bool LDS_LOOKUP>
__global__ __launch_bounds__(SS_COPY_THREADS) void ss_copy_kernel(
    uint8_t *__restrict__ arena, uint8_t *__restrict__ staging, const ss_desc_t *__restrict__ descs,
    const uint32_t *__restrict__ chunk0, const uint32_t *__restrict__ chunk_desc, uint32_t n_chunks,
    uint32_t chunk_shift, uint32_t n_desc) {
  const uint32_t tid = threadIdx.x;
  __shared__ uint32_t prefix[LDS_LOOKUP ? kLdsPrefixMax : 1];
  if (LDS_LOOKUP) {                               // n_desc + 1 <= kLdsPrefixMax is the launcher's business
    for (uint32_t i = tid; i <= n_desc; i += SS_COPY_THREADS) prefix[i] = chunk0[i];
    __syncthreads();
  }
  BlockWalk<TO_HOST, kUnroll, LDS_LOOKUP> w;
  w.arena = arena; w.staging = staging; w.descs = descs; w.chunk0 = chunk0; w.chunk_desc = chunk_desc;
  w.lds_prefix = prefix; w.n_desc = n_desc;
  w.n_chunks = n_chunks; w.chunk_shift = chunk_shift;
  w.c = blockIdx.x;
  if (!w.open_chunk()) return;
  CopyBlock cur, nxt;
  if (!w.next(cur)) return;
  u32x4 a[kUnroll], b[kUnroll];
  uint8_t ta = 0, tb = 0;
#pragma unroll
  for (uint32_t u = 0; u < kUnroll; ++u) {
    const uint32_t i = u * SS_COPY_THREADS + tid;
    if (i < cur.n16) a[u] = __builtin_nontemporal_load(cur.src + i);
  }
  if (tid < cur.tail) ta = reinterpret_cast<const uint8_t *>(cur.src + cur.n16)[tid];
  for (;;) {
    const bool more = w.next(nxt);
    if (more) {
#pragma unroll
      for (uint32_t u = 0; u < kUnroll; ++u) {
        const uint32_t i = u * SS_COPY_THREADS + tid;
        if (i < nxt.n16) b[u] = __builtin_nontemporal_load(nxt.src + i);
      }
      if (tid < nxt.tail) tb = reinterpret_cast<const uint8_t *>(nxt.src + nxt.n16)[tid];
    }
#pragma unroll
    for (uint32_t u = 0; u < kUnroll; ++u) {
      const uint32_t i = u * SS_COPY_THREADS + tid;
      if (i < cur.n16) __builtin_nontemporal_store(a[u], cur.dst + i);
    }
    if (tid < cur.tail) reinterpret_cast<uint8_t *>(cur.dst + cur.n16)[tid] = ta;
    if (!more) break;
#pragma unroll
    for (uint32_t u = 0; u < kUnroll; ++u) a[u] = b[u];
    ta = tb;
    cur = nxt;
  }
}

// One tensor given by its two addresses (no descriptor table): for batches whose device addresses arrive with
// the call.  Chunks of 64 KiB are dealt round-robin to the workgroups; within a chunk every lane keeps kUnroll
// 16-byte loads in flight before it stores them; the last chunk ends with a byte tail.
template <uint32_t kUnroll>
__global__ __launch_bounds__(SS_COPY_THREADS) void ss_copy_flat_kernel(const uint8_t *__restrict__ src,
                                                                       uint8_t *__restrict__ dst, uint64_t nbytes) {
  const uint32_t tid = threadIdx.x;
  const uint64_t n_chunks = (nbytes + SS_CHUNK_BYTES - 1) >> SS_CHUNK_SHIFT;
  for (uint64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const uint64_t off = c << SS_CHUNK_SHIFT;
    const uint64_t left = nbytes - off;
    const uint32_t n = left < SS_CHUNK_BYTES ? (uint32_t)left : SS_CHUNK_BYTES;
    const u32x4 *s16 = reinterpret_cast<const u32x4 *>(src + off);
    u32x4 *d16 = reinterpret_cast<u32x4 *>(dst + off);
    const uint32_t n16 = n >> 4;
    for (uint32_t base = 0; base < n16; base += SS_COPY_THREADS * kUnroll) {
      u32x4 v[kUnroll];
#pragma unroll
      for (uint32_t u = 0; u < kUnroll; ++u) {
        const uint32_t i = base + u * SS_COPY_THREADS + tid;
        if (i < n16) v[u] = __builtin_nontemporal_load(s16 + i);
      }
#pragma unroll
      for (uint32_t u = 0; u < kUnroll; ++u) {
        const uint32_t i = base + u * SS_COPY_THREADS + tid;
        if (i < n16) __builtin_nontemporal_store(v[u], d16 + i);
      }
    }
    if (tid < (n & 15u)) dst[off + ((uint64_t)n16 << 4) + tid] = src[off + ((uint64_t)n16 << 4) + tid];
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

// Holds its stream until the sequence number at `flag` (device memory, written by a copy-engine transfer) has
// reached `want`.  One wave; its first lane polls with system-scope loads, which see what the copy engine wrote
// without a kernel boundary in between, and sleeps between polls so that it takes next to no issue slots from
// the waves beside it.  The wait is bounded: after `limit_ticks` of the 100 MHz wall clock the lane sets *gave_up
// (device memory) and *timeouts (pinned host memory, touched on this path only) and the kernel ends like any
// other; while *gave_up is set no later wait polls at all, so a transfer that never comes costs one limit, not
// one per wait.
__global__ void ss_wait_flag_kernel(const uint64_t *flag, uint64_t want, uint64_t limit_ticks, uint32_t *gave_up,
                                    uint32_t *timeouts) {
  if (threadIdx.x != 0) return;
  const uint64_t t0 = wall_clock64();
  while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) < want) {
    if (__hip_atomic_load(gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) return;
    if (wall_clock64() - t0 > limit_ticks) {
      __hip_atomic_store(gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(timeouts, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      return;
    }
    __builtin_amdgcn_s_sleep(32);
  }
}

// Stores `value` at `flag` (device memory): where the stream it runs on stands, for ss_wait_flag_kernel on another
// stream.  Everything enqueued before it on its stream has completed and is visible when the store is.
__global__ void ss_mark_kernel(uint64_t *flag, uint64_t value) {
  __hip_atomic_store(flag, value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace

void ss_launch_mark(hipStream_t s, uint64_t *flag, uint64_t value) {
  hipLaunchKernelGGL(ss_mark_kernel, dim3(1), dim3(1), 0, s, flag, value);
}

void ss_launch_wait_flag(hipStream_t s, const uint64_t *flag, uint64_t want, uint64_t limit_ticks, uint32_t *gave_up,
                         uint32_t *timeouts) {
  hipLaunchKernelGGL(ss_wait_flag_kernel, dim3(1), dim3(64), 0, s, flag, want, limit_ticks, gave_up, timeouts);
}

void ss_launch_copy(hipStream_t s, uint32_t workgroups, uint32_t unroll, bool to_host, uint8_t *arena,
                    uint8_t *staging, const ss_desc_t *d_descs, const uint32_t *d_chunk0,
                    const uint32_t *d_chunk_desc, uint32_t n_chunks, uint32_t chunk_shift, uint32_t n_desc,
                    bool lds_lookup) {
  if (n_chunks == 0) return;
  const dim3 grid(workgroups < n_chunks ? workgroups : n_chunks), block(SS_COPY_THREADS);
  if (lds_lookup && n_desc != 0 && n_desc + 1 <= kLdsPrefixMax) {      // a batch too long for LDS takes the table
    if (to_host)
      hipLaunchKernelGGL((ss_copy_kernel<true, 8, true>), grid, block, 0, s, arena, staging, d_descs, d_chunk0,
                         d_chunk_desc, n_chunks, chunk_shift, n_desc);
    else
      hipLaunchKernelGGL((ss_copy_kernel<false, 8, true>), grid, block, 0, s, arena, staging, d_descs, d_chunk0,
                         d_chunk_desc, n_chunks, chunk_shift, n_desc);
    return;
  }
#define SS_LAUNCH(TH, U)                                                                                  \
  hipLaunchKernelGGL((ss_copy_kernel<TH, U, false>), grid, block, 0, s, arena, staging, d_descs, d_chunk0, \
                     d_chunk_desc, n_chunks, chunk_shift, n_desc)
  if (to_host) {
    if (unroll <= 2) SS_LAUNCH(true, 2); else if (unroll <= 4) SS_LAUNCH(true, 4); else SS_LAUNCH(true, 8);
  } else {
    if (unroll <= 2) SS_LAUNCH(false, 2); else if (unroll <= 4) SS_LAUNCH(false, 4); else SS_LAUNCH(false, 8);
  }
#undef SS_LAUNCH
}

void ss_launch_copy_flat(hipStream_t s, uint32_t workgroups, const uint8_t *src, uint8_t *dst, uint64_t nbytes) {
  if (nbytes == 0) return;
  const uint64_t n_chunks = (nbytes + SS_CHUNK_BYTES - 1) >> SS_CHUNK_SHIFT;
  const dim3 grid((uint32_t)(workgroups < n_chunks ? workgroups : n_chunks)), block(SS_COPY_THREADS);
  hipLaunchKernelGGL((ss_copy_flat_kernel<8>), grid, block, 0, s, src, dst, nbytes);
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
