// Sequence aligner: longest common subsequence of the reference and the current operator sequence
// and the canonical alignment read off it; the matcher's fourth level (Sec. 5.1 asks for tolerance
// to minor sequence variations with integer-only comparison and gives no algorithm).
//
// The dynamic programme runs in its bit-vector form on one wavefront: bit j of V_i is 0 exactly
// when L[i][j+1] = L[i][j] + 1, V_0 is all ones, and one reference operator advances the row by
//     V' = (V + (V & M)) | (V & ~M),     M = positions of cur holding that operator's key.
// A row of m bits lives in the registers of 64 lanes (K 64-bit words each, lane l owning words
// l*K .. l*K+K-1); the addition's carries cross lanes through two ballots: with G = lanes whose
// words overflow on their own and P = lanes whose words are all ones, the carry into lane l is bit
// l of P ^ ((G | P) + G).  Every row is written out; the host walks back from (n, m): equal
// operators pair, otherwise left if bit j-1 of V_i is set (L[i][j-1] = L[i][j]), else up.
#include <algorithm>
#include <cstring>
#include <unordered_map>

#include "ss_internal.h"

namespace {

constexpr uint32_t kAlignLenLimit = 1u << 16;          // 16 words per lane
constexpr size_t kAlignRowBytesLimit = 1ull << 30;     // rows kept for the walk back
constexpr size_t kLdsMaskBytes = 48 * 1024;

__global__ void ss_align_masks_kernel(const uint32_t *__restrict__ cur_id, uint32_t m,
                                      unsigned long long *__restrict__ masks, uint32_t W) {
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < m) atomicOr(&masks[(size_t)cur_id[j] * W + (j >> 6)], 1ull << (j & 63));
}

template <int K, bool LDS>
__global__ __launch_bounds__(64) void ss_align_rows_kernel(const uint32_t *__restrict__ ref_id, uint32_t n,
                                                           const unsigned long long *__restrict__ masks,
                                                           uint32_t W, uint32_t n_mask_rows,
                                                           unsigned long long *__restrict__ rows) {
  extern __shared__ unsigned long long lds_masks[];
  const uint32_t lane = threadIdx.x;
  if (LDS) {
    for (uint32_t idx = lane; idx < n_mask_rows * W; idx += 64) lds_masks[idx] = masks[idx];
    __syncthreads();
  }
  const unsigned long long *table = LDS ? lds_masks : masks;
  const uint32_t w0 = lane * K;
  unsigned long long V[K], Mn[K];
#pragma unroll
  for (int k = 0; k < K; ++k) V[k] = ~0ull;

  auto load_masks = [&](uint32_t id, unsigned long long *M) {
    const unsigned long long *mrow = table + (size_t)id * W;
#pragma unroll
    for (int k = 0; k < K; ++k) M[k] = (w0 + k < W) ? mrow[w0 + k] : 0ull;
  };

  for (uint32_t i0 = 0; i0 < n; i0 += 64) {
    const uint32_t cnt = min(64u, n - i0);
    const uint32_t my_id = (lane < cnt) ? ref_id[i0 + lane] : 0u;
    load_masks(__shfl(my_id, 0), Mn);
    for (uint32_t r = 0; r < cnt; ++r) {
      unsigned long long M[K], S[K];
#pragma unroll
      for (int k = 0; k < K; ++k) M[k] = Mn[k];
      if (r + 1 < cnt) load_masks(__shfl(my_id, r + 1), Mn);   // next row's masks fly while this row adds
      unsigned long long carry = 0;
      bool ones = true;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const unsigned long long U = V[k] & M[k];
        const unsigned long long t = V[k] + U;
        unsigned long long c = t < U ? 1ull : 0ull;
        const unsigned long long s = t + carry;
        c |= s < t ? 1ull : 0ull;
        S[k] = s;
        carry = c;
        ones = ones && (s == ~0ull);
      }
      const unsigned long long G = __ballot(carry != 0), P = __ballot(ones);
      const unsigned long long cin_all = P ^ ((G | P) + G);
      unsigned long long cin = (cin_all >> lane) & 1ull;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        S[k] += cin;
        cin = cin & (S[k] == 0ull ? 1ull : 0ull);
        V[k] = S[k] | (V[k] & ~M[k]);
        if (w0 + k < W) rows[(size_t)(i0 + r) * W + w0 + k] = V[k];
      }
    }
  }
}

struct KeyHash {
  size_t operator()(const std::pair<uint64_t, uint32_t> &k) const {
    uint64_t x = k.first * 0x9E3779B97F4A7C15ull ^ ((uint64_t)k.second * 0xC2B2AE3D27D4EB4Full);
    x ^= x >> 29;
    return (size_t)x;
  }
};

template <int K>
void launch_rows(hipStream_t s, bool lds, size_t lds_bytes, const uint32_t *ref_id, uint32_t n,
                 const unsigned long long *masks, uint32_t W, uint32_t n_mask_rows, unsigned long long *rows) {
  if (lds)
    hipLaunchKernelGGL((ss_align_rows_kernel<K, true>), dim3(1), dim3(64), lds_bytes, s, ref_id, n, masks, W,
                       n_mask_rows, rows);
  else
    hipLaunchKernelGGL((ss_align_rows_kernel<K, false>), dim3(1), dim3(64), 0, s, ref_id, n, masks, W,
                       n_mask_rows, rows);
}

}  // namespace

// ref_to_cur: n entries (host), filled; *lcs out.  Shared by ss_align_sequence and the SS_MATCH_ALIGN
// branch of ss_match_sequence.
int ss_align_core(ss_ctx *ctx, const ss_op_t *ref, uint32_t n, const ss_op_t *cur, uint32_t m,
                  int32_t *ref_to_cur, uint32_t *lcs, uint32_t *n_keys_out) {
  if (n > kAlignLenLimit || m > kAlignLenLimit) return SS_E_CAPACITY;
  for (uint32_t i = 0; i < n; ++i) ref_to_cur[i] = -1;
  *lcs = 0;
  if (n_keys_out) *n_keys_out = 0;
  if (n == 0 || m == 0) return SS_OK;

  // dense key ids: the keys of cur in first-seen order; reference operators whose key cur does not
  // hold share the id n_keys, whose mask row stays zero
  std::unordered_map<std::pair<uint64_t, uint32_t>, uint32_t, KeyHash> ids;
  ids.reserve(256);
  std::vector<uint32_t> cur_id(m), ref_id(n);
  for (uint32_t j = 0; j < m; ++j) {
    const std::pair<uint64_t, uint32_t> key{((uint64_t)cur[j].op_token << 32) | cur[j].stack_hash, cur[j].sig};
    auto it = ids.find(key);
    if (it == ids.end()) it = ids.emplace(key, (uint32_t)ids.size()).first;
    cur_id[j] = it->second;
  }
  const uint32_t n_keys = (uint32_t)ids.size();
  for (uint32_t i = 0; i < n; ++i) {
    const std::pair<uint64_t, uint32_t> key{((uint64_t)ref[i].op_token << 32) | ref[i].stack_hash, ref[i].sig};
    auto it = ids.find(key);
    ref_id[i] = it == ids.end() ? n_keys : it->second;
  }
  if (n_keys_out) *n_keys_out = n_keys;

  const uint32_t W = (m + 63) / 64;
  const size_t mask_bytes = (size_t)(n_keys + 1) * W * 8, row_bytes = (size_t)n * W * 8;
  if (row_bytes > kAlignRowBytesLimit || mask_bytes > kAlignRowBytesLimit) return SS_E_CAPACITY;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += ss_align_up(bytes, 256); return o; };
  const size_t o_ref = take((size_t)n * 4), o_cur = take((size_t)m * 4), o_mask = take(mask_bytes),
               o_rows = take(row_bytes);
  int rc = ss_scratch_reserve(ctx, off, row_bytes);
  if (rc != SS_OK) return rc;
  uint8_t *d = (uint8_t *)ctx->d_scratch;
  hipStream_t s = ctx->s_aux;
  SS_HIP(hipMemcpyAsync(d + o_ref, ref_id.data(), (size_t)n * 4, hipMemcpyHostToDevice, s));
  SS_HIP(hipMemcpyAsync(d + o_cur, cur_id.data(), (size_t)m * 4, hipMemcpyHostToDevice, s));
  ss_launch_fill(s, d + o_mask, mask_bytes, 0);
  unsigned long long *masks = (unsigned long long *)(d + o_mask), *rows = (unsigned long long *)(d + o_rows);
  hipLaunchKernelGGL(ss_align_masks_kernel, dim3((m + 255) / 256), dim3(256), 0, s, (const uint32_t *)(d + o_cur), m,
                     masks, W);
  const bool lds = mask_bytes <= kLdsMaskBytes;
  const uint32_t k_words = (W + 63) / 64;                 // words per lane, rounded up to 1, 2, 4, 8, 16
  const uint32_t *dref = (const uint32_t *)(d + o_ref);
  if (k_words <= 1) launch_rows<1>(s, lds, mask_bytes, dref, n, masks, W, n_keys + 1, rows);
  else if (k_words <= 2) launch_rows<2>(s, lds, mask_bytes, dref, n, masks, W, n_keys + 1, rows);
  else if (k_words <= 4) launch_rows<4>(s, lds, mask_bytes, dref, n, masks, W, n_keys + 1, rows);
  else if (k_words <= 8) launch_rows<8>(s, lds, mask_bytes, dref, n, masks, W, n_keys + 1, rows);
  else launch_rows<16>(s, lds, mask_bytes, dref, n, masks, W, n_keys + 1, rows);
  SS_HIP(hipGetLastError());
  const uint64_t *h = (const uint64_t *)ctx->h_scratch;
  SS_HIP(hipMemcpyAsync(ctx->h_scratch, rows, row_bytes, hipMemcpyDeviceToHost, s));
  SS_HIP(hipStreamSynchronize(s));

  // walk back from (n, m); row i of the table is h[(i - 1) * W ..]
  uint32_t i = n, j = m, pairs = 0;
  while (i > 0 && j > 0) {
    if (ref_id[i - 1] == cur_id[j - 1]) {
      ref_to_cur[i - 1] = (int32_t)(j - 1);
      ++pairs;
      --i;
      --j;
    } else if ((h[(size_t)(i - 1) * W + ((j - 1) >> 6)] >> ((j - 1) & 63)) & 1ull) {
      --j;
    } else {
      --i;
    }
  }
  *lcs = pairs;
  return SS_OK;
}

void ss_align_anchors(const ss_op_t *ref, uint32_t n, const ss_op_t *cur, const int32_t *ref_to_cur,
                      const ss_anchor_t *anchors, uint32_t k, int32_t *new_idx, uint8_t *level,
                      uint32_t *n_unmatched) {
  (void)ref;
  uint32_t unm = 0;
  for (uint32_t a = 0; a < k; ++a) {
    const uint32_t i = anchors[a].ref_op;
    int32_t j = -1;
    if (i < n && ref_to_cur[i] >= 0 && anchors[a].out_slot < cur[ref_to_cur[i]].n_out) j = ref_to_cur[i];
    new_idx[a] = j;
    level[a] = j >= 0 ? (uint8_t)SS_LEVEL_ALIGN : (uint8_t)255;
    unm += j < 0;
  }
  *n_unmatched = unm;
}

extern "C" int ss_align_sequence(ss_ctx *ctx, const ss_op_t *ref, uint32_t n_ref, const ss_op_t *cur,
                                 uint32_t n_cur, const ss_anchor_t *anchors, uint32_t n_anchors,
                                 int32_t *ref_to_cur, int32_t *new_idx, uint8_t *level, ss_align_result_t *res) {
  return ss_guard([&]() -> int {
    if (!ctx || !res || (n_ref && !ref) || (n_cur && !cur)) return SS_E_INVAL;
    if (n_anchors && (!anchors || !new_idx || !level)) return SS_E_INVAL;
    std::vector<int32_t> local;
    if (!ref_to_cur) {
      local.resize(n_ref);
      ref_to_cur = local.data();
    }
    std::memset(res, 0, sizeof(*res));
    uint32_t lcs = 0, n_keys = 0;
    int rc = ss_align_core(ctx, ref, n_ref, cur, n_cur, ref_to_cur, &lcs, &n_keys);
    if (rc != SS_OK) return rc;
    res->lcs = lcs;
    res->distance = n_ref + n_cur - 2 * lcs;
    res->n_keys = n_keys;
    ss_align_anchors(ref, n_ref, cur, ref_to_cur, anchors, n_anchors, new_idx, level, &res->n_unmatched);
    for (uint32_t a = 0; a < n_anchors; ++a) ctx->stats.match_levels[level[a] <= SS_LEVEL_ALIGN ? level[a] : 4]++;
    return SS_OK;
  });
}
