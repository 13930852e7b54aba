// pfc_sample: the sampled class set S of one iteration (arXiv 2203.15565, Sec. 3.2 / Fig. 4:
// the classes present in the batch go in first, random negatives fill the buffer up to r*N).
//
// Integer work only.  Every class gets a 32-bit Philox4x32-10 score (Salmon et al., SC'11),
// recomputed wherever it is needed (about 60 integer operations per four classes; nothing is
// stored per class except one "is in the batch" bit).  The k - U negatives with the largest
// scores are found by a three-pass radix select (8 + 12 + 12 bits), equal scores going to the
// smaller class id; an index-ordered compaction then writes S in ascending class id.
#include <math.h>
#include <string.h>

#include <mutex>

#include "pfc_common.h"

namespace pfc {

namespace {

constexpr int kThreads = 256;
constexpr int kClassesPerBlock = 2048;                 // ordered passes: 2 x (256 threads x 4)
constexpr int kItersPerBlock = kClassesPerBlock / (kThreads * 4);

// Radix passes over the 32-bit score: bits [31:24], [23:12], [11:0].  The first pass sees every
// class, so it is kept narrow (256 bins: few global atomics per block); the later passes see
// only the classes inside the chosen bin, so their 4096-bin histograms are almost empty.
constexpr int kHistStride = 4096;
template <int P> struct Pass;
template <> struct Pass<0> { static constexpr int kBins = 256, kShift = 24; };
template <> struct Pass<1> { static constexpr int kBins = 4096, kShift = 12; };
template <> struct Pass<2> { static constexpr int kBins = 4096, kShift = 0; };

struct PhiloxKey {
  uint32_t k0, k1;   // lo32(seed), hi32(seed)
  uint32_t c2, c3;   // lo32(step), hi32(step)
  uint32_t mask;     // ANDed onto every score
};

// Scores of classes 4q .. 4q+3.
__device__ __forceinline__ void philox_block(uint32_t q, const PhiloxKey& key, uint32_t out[4]) {
  uint32_t c0 = q, c1 = 0u, c2 = key.c2, c3 = key.c3;   // class ids are < 2^31, so hi32(j/4) = 0
  uint32_t k0 = key.k0, k1 = key.k1;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0 & key.mask; out[1] = c1 & key.mask; out[2] = c2 & key.mask; out[3] = c3 & key.mask;
}

// The four "is positive" bits of classes 4q..4q+3 (bit e = class 4q+e).
__device__ __forceinline__ uint32_t pos_nibble(const uint32_t* __restrict__ pos_bits, uint32_t q) {
  return (pos_bits[q >> 3] >> ((q & 7u) * 4u)) & 0xFu;
}

// Between two calls the sampler's scratch is all zero (bitmap, histograms, counter of positives):
// pfc_create clears it once, and the last reader of each piece clears it again -- the scan of a
// pass its histogram, the first scan the counter, the label remap the bitmap words it knows to be
// set -- so no call starts with a clearing pass.  The batch classes are marked inside the launch
// of the first radix pass (see sample_hist_kernel), not by a launch of their own.

// All 256 threads of a workgroup: walk the merged histogram of pass P from the largest bin
// downwards until `need` classes are covered.  Returns (to every thread) the bin that holds the
// threshold and how many classes are still to be taken from inside it.  Every workgroup of the
// launch that follows pass P does this for itself -- the same integers everywhere -- instead of a
// one-workgroup launch in between.
template <int P>
__device__ __forceinline__ void find_bin(const uint32_t* __restrict__ hist, uint32_t need,
                                         uint32_t& bin, uint32_t& need_inside) {
  __shared__ uint32_t wsum[4];
  __shared__ uint32_t s_bin, s_need;
  constexpr int kBins = Pass<P>::kBins;
  constexpr int kPer = kBins / kThreads;
  const int t = threadIdx.x;
  // thread t owns the descending bins kBins-1-t*kPer .. kBins-1-(t*kPer+kPer-1)
  uint32_t own[kPer];
  uint32_t mine = 0;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    own[e] = hist[P * kHistStride + (kBins - 1 - (t * kPer + e))];
    mine += own[e];
  }
  uint32_t inc = mine;   // inclusive scan over threads
  const int lane = t & 63, w = t >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t n = __shfl_up(inc, o, 64);
    if (lane >= o) inc += n;
  }
  if (lane == 63) wsum[w] = inc;
  if (t == 0) {
    s_bin = 0u;
    s_need = 0u;
  }
  __syncthreads();
  uint32_t base = 0;
  for (int i = 0; i < w; ++i) base += wsum[i];
  inc += base;
  const uint32_t exc = inc - mine;
  if (exc < need && need <= inc) {   // true in exactly one thread (if need >= 1)
    uint32_t cum = exc;
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      if (cum + own[e] >= need) {
        s_bin = (uint32_t)(kBins - 1 - (t * kPer + e));
        s_need = need - cum;
        break;
      }
      cum += own[e];
    }
  }
  __syncthreads();
  bin = s_bin;
  need_inside = s_need;
  __syncthreads();
}

// State of the select after pass P-1, found by every workgroup of the launch of pass P (or of the
// count launch, P = 3) from the histogram of pass P-1 and what workgroup 0 of the launch before
// left in `sel`.  Workgroup 0 records the new state for the next launch and clears what nobody
// reads any more (the histogram of pass P-2, the count of positives).
template <int P>
__device__ __forceinline__ void select_state(uint32_t* __restrict__ hist, SelState* __restrict__ sel,
                                             uint32_t ceil_rN, uint32_t& prefix, uint32_t& need,
                                             uint32_t& none) {
  static_assert(P >= 1 && P <= 3, "state after pass P-1");
  uint32_t need_in, prefix_in;
  if constexpr (P == 1) {
    const uint32_t U = sel->U;
    const uint32_t k = U > ceil_rN ? U : ceil_rN;
    none = (k == U) ? 1u : 0u;
    need_in = k - U;
    prefix_in = 0u;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      sel->k = k;
      sel->none = none;
    }
  } else {
    none = sel->none;
    need_in = sel->need[P - 2];
    prefix_in = sel->prefix[P - 2];
  }
  uint32_t bin = 0u;
  need = 0u;
  if (!none) find_bin<P - 1>(hist, need_in, bin, need);
  prefix = prefix_in | (bin << Pass<P - 1>::kShift);
  if (blockIdx.x == 0) {
    if (threadIdx.x == 0) {
      sel->need[P - 1] = need;
      sel->prefix[P - 1] = prefix;
      if (P == 2) sel->U = 0u;
    }
    if constexpr (P >= 2) {
      constexpr int kOld = Pass<P - 2>::kBins;
      for (int b = threadIdx.x; b < kOld; b += kThreads) hist[(P - 2) * kHistStride + b] = 0u;
    }
  }
}

// Radix pass P over the classes whose score agrees with the prefix found so far.
// Passes 1 and 2 skip the classes of the batch (their bits are complete by then).  Pass 0 runs in
// the same launch as the marking of the batch classes, so it cannot know them yet: it counts EVERY
// class, and the workgroups behind the first `hist_blocks` mark the labels -- the one thread that
// sets a class's bit first takes that class's score out of the merged histogram again and counts
// the class as a positive.  Integer atomics only, so the histogram after the launch is the same
// whatever the order.
template <int P>
__global__ void sample_hist_kernel(int64_t N, PhiloxKey key, uint32_t* __restrict__ pos_bits,
                                   uint32_t* __restrict__ hist, SelState* __restrict__ sel,
                                   uint32_t ceil_rN, const int64_t* __restrict__ labels, int B,
                                   int hist_blocks, int32_t* __restrict__ err_flag) {
  constexpr int kBins = Pass<P>::kBins, kShift = Pass<P>::kShift;
  if constexpr (P == 0) {
    if ((int)blockIdx.x >= hist_blocks) {   // marking part of the launch
      const int i = ((int)blockIdx.x - hist_blocks) * kThreads + threadIdx.x;
      const int64_t y = i < B ? labels[i] : 0;
      const bool valid = i < B && y >= 0 && y < N;
      if (i < B && !valid) atomicOr(err_flag, 1);
      // One lane per distinct label of the wavefront goes on: with long-tailed labels a frequent
      // class would otherwise bring thousands of atomics onto one word.
      bool lead = false;
      unsigned long long todo = __ballot(valid);
      while (todo) {   // wave-uniform loop over the distinct labels
        const int src = __ffsll(todo) - 1;
        const int64_t y0 = __shfl(y, src, 64);
        lead = lead || (int)(threadIdx.x & 63) == src;
        todo &= ~__ballot(valid && y == y0);
      }
      if (!lead) return;
      const uint32_t bit = 1u << (y & 31);
      const uint32_t old = atomicOr(&pos_bits[y >> 5], bit);
      if (!(old & bit)) {   // first to mark class y
        uint32_t u[4];
        philox_block((uint32_t)(y >> 2), key, u);
        atomicSub(&hist[u[y & 3] >> kShift], 1u);
        atomicAdd(&sel->U, 1u);
      }
      return;
    }
  }
  __shared__ uint32_t lh[kBins];
  for (int b = threadIdx.x; b < kBins; b += blockDim.x) lh[b] = 0u;
  uint32_t prefix = 0u, need = 0u, none = 0u;
  if constexpr (P > 0) select_state<P>(hist, sel, ceil_rN, prefix, need, none);
  __syncthreads();
  if (!(P > 0 && none)) {
    const uint32_t nq = (uint32_t)((N + 3) >> 2);
    const uint32_t stride = (uint32_t)hist_blocks * blockDim.x;
    for (uint32_t q = blockIdx.x * blockDim.x + threadIdx.x; q < nq; q += stride) {
      uint32_t u[4];
      philox_block(q, key, u);
      uint32_t pb = 0u;
      if constexpr (P > 0) pb = pos_nibble(pos_bits, q);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int64_t j = (int64_t)q * 4 + e;
        if (j >= N || ((pb >> e) & 1u)) continue;
        if (P == 0) {
          atomicAdd(&lh[u[e] >> kShift], 1u);
        } else {
          // bits above this pass's field must equal the prefix
          constexpr int kAbove = kShift + 12;
          if ((u[e] >> kAbove) == (prefix >> kAbove))
            atomicAdd(&lh[(u[e] >> kShift) & (kBins - 1)], 1u);
        }
      }
    }
  }
  __syncthreads();
  for (int b = threadIdx.x; b < kBins; b += blockDim.x) {
    const uint32_t c = lh[b];
    if (c) atomicAdd(&hist[P * kHistStride + b], c);
  }
}

// Selection predicate pieces for classes 4q..4q+3: bit e of `sure` = positive or score above the
// threshold; bit e of `eq` = non-positive and score equal to the threshold.
__device__ __forceinline__ void classify(uint32_t q, int64_t N, const PhiloxKey& key,
                                         const uint32_t* __restrict__ pos_bits, uint32_t T,
                                         uint32_t none, uint32_t& sure, uint32_t& eq) {
  sure = 0u;
  eq = 0u;
  const uint32_t nq = (uint32_t)((N + 3) >> 2);
  if (q >= nq) return;
  uint32_t u[4];
  philox_block(q, key, u);
  const uint32_t pb = pos_nibble(pos_bits, q);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int64_t j = (int64_t)q * 4 + e;
    if (j >= N) continue;
    if ((pb >> e) & 1u) {
      sure |= 1u << e;
    } else if (!none) {
      if (u[e] > T) sure |= 1u << e;
      else if (u[e] == T) eq |= 1u << e;
    }
  }
}

__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t* sm) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  const uint32_t r = sm[0] + sm[1] + sm[2] + sm[3];
  __syncthreads();
  return r;
}

// exclusive scan over the 256 threads of a block; also returns the block total
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* sm, uint32_t& total) {
  uint32_t inc = v;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t n = __shfl_up(inc, o, 64);
    if (lane >= o) inc += n;
  }
  if (lane == 63) sm[w] = inc;
  __syncthreads();
  uint32_t base = 0;
  for (int i = 0; i < w; ++i) base += sm[i];
  total = sm[0] + sm[1] + sm[2] + sm[3];
  __syncthreads();
  return base + inc - v;
}

__global__ void sample_count_kernel(int64_t N, PhiloxKey key, const uint32_t* __restrict__ pos_bits,
                                    uint32_t* __restrict__ hist, SelState* __restrict__ sel,
                                    uint32_t ceil_rN, uint32_t* __restrict__ blk_cnt) {
  __shared__ uint32_t sm[4];
  uint32_t T, need, none;
  select_state<3>(hist, sel, ceil_rN, T, need, none);   // the full 32-bit threshold
  uint32_t nsure = 0, neq = 0;
#pragma unroll
  for (int it = 0; it < kItersPerBlock; ++it) {
    const uint32_t q = blockIdx.x * (kClassesPerBlock / 4) + it * kThreads + threadIdx.x;
    uint32_t sure, eq;
    classify(q, N, key, pos_bits, T, none, sure, eq);
    nsure += __popc(sure);
    neq += __popc(eq);
  }
  const uint32_t bs = block_sum(nsure, sm);
  const uint32_t be = block_sum(neq, sm);
  if (threadIdx.x == 0) {
    blk_cnt[2 * blockIdx.x] = bs;
    blk_cnt[2 * blockIdx.x + 1] = be;
  }
}

// Ordered write of S.  Every block first adds up the counts of the blocks in front of it: its
// output offset is their "sure" classes plus the equal-to-threshold ones they were allowed to
// keep -- the quota sel->need is used up in ascending class id, so that is min(quota, number of
// equal classes in front).  The last block also leaves the total in sel->total.
__global__ void sample_write_kernel(int64_t N, PhiloxKey key, const uint32_t* __restrict__ pos_bits,
                                    SelState* __restrict__ sel, uint32_t* __restrict__ hist,
                                    const uint32_t* __restrict__ blk_cnt, int64_t cap,
                                    int32_t* __restrict__ idx_out) {
  __shared__ uint32_t sm[4];
  const uint32_t T = sel->prefix[2], none = sel->none;
  const uint32_t need_eq = none ? 0u : sel->need[2];
  if (blockIdx.x == 0)   // nobody reads the last pass's histogram any more
    for (int b = threadIdx.x; b < Pass<2>::kBins; b += kThreads) hist[2 * kHistStride + b] = 0u;
  uint32_t front_sure = 0, front_eq = 0;
  for (uint32_t b = threadIdx.x; b < blockIdx.x; b += kThreads) {
    front_sure += blk_cnt[2 * b];
    front_eq += blk_cnt[2 * b + 1];
  }
  front_sure = block_sum(front_sure, sm);
  front_eq = block_sum(front_eq, sm);
  uint32_t out = front_sure + (front_eq < need_eq ? front_eq : need_eq);
  uint32_t eq_run = front_eq;
#pragma unroll
  for (int it = 0; it < kItersPerBlock; ++it) {
    const uint32_t q = blockIdx.x * (kClassesPerBlock / 4) + it * kThreads + threadIdx.x;
    uint32_t sure, eq;
    classify(q, N, key, pos_bits, T, none, sure, eq);
    uint32_t tot_e, tot_s;
    uint32_t eq_rank = eq_run + block_excl_scan(__popc(eq), sm, tot_e);
    // keep an equal-score class only while the quota lasts (ascending class id)
    uint32_t chosen = sure;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if ((eq >> e) & 1u) {
        if (eq_rank < need_eq) chosen |= 1u << e;
        ++eq_rank;
      }
    }
    uint32_t pos = out + block_excl_scan(__popc(chosen), sm, tot_s);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if ((chosen >> e) & 1u) {
        if ((int64_t)pos < cap) idx_out[pos] = (int32_t)(q * 4u + e);
        ++pos;
      }
    }
    eq_run += tot_e;
    out += tot_s;
  }
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) sel->total = out;
}

// labels_local[i] = position of labels[i] in the ascending idx (binary search), -1 if absent.
__global__ void sample_remap_kernel(const int64_t* __restrict__ labels, int B, int64_t N,
                                    const int32_t* __restrict__ idx, const SelState* __restrict__ sel,
                                    int64_t cap, int32_t* __restrict__ yl_out,
                                    uint32_t* __restrict__ pos_bits) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B) return;
  const int64_t y = labels[i];
  int64_t k = sel->total;
  if (k > cap) k = cap;
  int32_t res = -1;
  if (y >= 0 && y < N) {
    int64_t lo = 0, hi = k;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if (idx[mid] < (int32_t)y) lo = mid + 1; else hi = mid;
    }
    if (lo < k && idx[lo] == (int32_t)y) res = (int32_t)lo;
  }
  yl_out[i] = res;
  // last user of the "is in the batch" bits: clear this label's word for the next call
  if (y >= 0 && y < N) pos_bits[y >> 5] = 0u;
}

}  // namespace

int sample_impl(pfc_ctx* c, const int64_t* labels, int32_t B, double r, uint64_t seed,
                uint64_t step, uint32_t score_mask, int32_t* idx_out, int32_t* yl_out,
                int64_t* k_out) {
  const int64_t N = c->N;
  int64_t crn = (int64_t)ceil(r * (double)N);
  if (crn > N) crn = N;
  if (crn < 1) crn = 1;
  const int64_t cap = pfc_num_sampled(N, B, r);
  PhiloxKey key;
  key.k0 = (uint32_t)(seed & 0xFFFFFFFFu);
  key.k1 = (uint32_t)(seed >> 32);
  key.c2 = (uint32_t)(step & 0xFFFFFFFFu);
  key.c3 = (uint32_t)(step >> 32);
  key.mask = score_mask;

  const int nblk = (int)((N + kClassesPerBlock - 1) / kClassesPerBlock);
  if (nblk > c->nblk_cap) return PFC_EINVAL;
  const int64_t nq = (N + 3) / 4;
  int hist_blocks = (int)((nq + kThreads * 4 - 1) / (kThreads * 4));
  if (hist_blocks > 512) hist_blocks = 512;
  if (hist_blocks < 1) hist_blocks = 1;

  const int mark_blocks = (B + kThreads - 1) / kThreads;
  PFC_LAUNCH(c, KID_SAMPLE_HIST0, sample_hist_kernel<0>, dim3(hist_blocks + mark_blocks),
             dim3(kThreads), 0, N, key, c->pos_bits, c->hist, c->sel, (uint32_t)crn, labels, B,
             hist_blocks, c->err_flag);
  PFC_LAUNCH(c, KID_SAMPLE_HIST1, sample_hist_kernel<1>, dim3(hist_blocks), dim3(kThreads), 0, N,
             key, c->pos_bits, c->hist, c->sel, (uint32_t)crn, labels, B, hist_blocks, c->err_flag);
  PFC_LAUNCH(c, KID_SAMPLE_HIST2, sample_hist_kernel<2>, dim3(hist_blocks), dim3(kThreads), 0, N,
             key, c->pos_bits, c->hist, c->sel, (uint32_t)crn, labels, B, hist_blocks, c->err_flag);
  PFC_LAUNCH(c, KID_SAMPLE_COUNT, sample_count_kernel, dim3(nblk), dim3(kThreads), 0, N, key,
             c->pos_bits, c->hist, c->sel, (uint32_t)crn, c->blk_cnt);
  PFC_LAUNCH(c, KID_SAMPLE_WRITE, sample_write_kernel, dim3(nblk), dim3(kThreads), 0, N, key,
             c->pos_bits, c->sel, c->hist, c->blk_cnt, cap, idx_out);
  PFC_LAUNCH(c, KID_SAMPLE_REMAP, sample_remap_kernel, dim3((B + kThreads - 1) / kThreads),
             dim3(kThreads), 0, labels, B, N, idx_out, c->sel, cap, yl_out, c->pos_bits);

  if (crn >= (int64_t)B) {
    // U <= B <= ceil(r*N): k is known without the labels.
    *k_out = crn;
  } else {
    PFC_HIP(hipMemcpyAsync(c->host_pin, &c->sel->k, 4, hipMemcpyDeviceToHost, c->stream));
    PFC_HIP(hipStreamSynchronize(c->stream));
    *k_out = (int64_t)c->host_pin[0];
  }
  return PFC_OK;
}

}  // namespace pfc

// ---------------------------------------------------------------------------------------------
// pfc_sample_noalloc: pfc_sample for callers that cannot allocate.  The sampler's scratch (the
// "is in the batch" bitmap, the radix histograms, the select state, the per-block counts and an
// error word) lives in ONE file-scope device array per GPU instead of a context's hipMalloc'ed
// buffers; the kernels are those of pfc_sample and take its pieces as pointers.
// ---------------------------------------------------------------------------------------------
namespace {

constexpr int64_t kNoallocMaxN = (int64_t)1 << 24;                               // 16,777,216 classes
constexpr size_t kNaBitmapWords = (size_t)(kNoallocMaxN / 32) + 64;              // as pfc_create sizes it
constexpr size_t kNaHistWords = 3 * 4096;
constexpr size_t kNaSelWords = 64;                                               // SelState, 256-byte slot
constexpr size_t kNaBlkWords = 2 * (size_t)(kNoallocMaxN / pfc::kClassesPerBlock);
constexpr size_t kNaErrWords = 64;
constexpr size_t kNaOffHist = kNaBitmapWords;
constexpr size_t kNaOffSel = kNaOffHist + kNaHistWords;
constexpr size_t kNaOffBlk = kNaOffSel + kNaSelWords;
constexpr size_t kNaOffErr = kNaOffBlk + kNaBlkWords;
constexpr size_t kNaWords = kNaOffErr + kNaErrWords;                             // 2.2 MB
static_assert(sizeof(pfc::SelState) <= kNaSelWords * 4, "select state slot");

// Zero when the code object is loaded; afterwards every call leaves it zero again (the last
// reader of each piece clears it, see above), except the error word, which only ever gains bits.
static __device__ __align__(256) uint32_t scratch[kNaWords];

constexpr int kNaMaxDevices = 64;
std::mutex g_na_mutex;
uint32_t* g_na_ptr[kNaMaxDevices];   // device address of `scratch` on each GPU, once looked up

// The array's name is only a host-side handle: its address on the current device comes from the
// runtime, once per device, and is what the kernels are given.
int noalloc_scratch(uint32_t** out) {
  int dev = -1;
  PFC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kNaMaxDevices) return PFC_EINVAL;
  std::lock_guard<std::mutex> lock(g_na_mutex);
  if (!g_na_ptr[dev]) {
    uint32_t* p = nullptr;
    PFC_HIP(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    if (!p) return PFC_EHIP;
    g_na_ptr[dev] = p;
  }
  *out = g_na_ptr[dev];
  return PFC_OK;
}

}  // namespace

extern "C" int pfc_sample_noalloc(const int64_t* labels, int32_t B, int64_t N, double r,
                                  uint64_t seed, uint64_t step, int32_t* idx_out,
                                  int32_t* labels_local_out, int64_t* k_out, void* hip_stream) {
  if (!labels || !idx_out || !labels_local_out || !k_out) return PFC_EINVAL;
  if (N < 1 || N > kNoallocMaxN) return PFC_EINVAL;
  if (B < 1 || B > (1 << 20)) return PFC_EINVAL;
  if (!(r > 0.0) || !(r <= 1.0)) return PFC_EINVAL;
  // k must be known without reading anything back: no waiting, no pinned buffer
  if ((int64_t)ceil(r * (double)N) < (int64_t)B) return PFC_EINVAL;
  uint32_t* base = nullptr;
  const int rc = noalloc_scratch(&base);
  if (rc != PFC_OK) return rc;
  pfc_ctx c;   // a view of the static scratch on the stack: nothing is allocated, nothing kept
  memset(&c, 0, sizeof(c));
  c.N = N;
  c.stream = (hipStream_t)hip_stream;
  c.pos_bits = base;
  c.hist = base + kNaOffHist;
  c.sel = reinterpret_cast<pfc::SelState*>(base + kNaOffSel);
  c.blk_cnt = base + kNaOffBlk;
  c.nblk_cap = (int32_t)(kNoallocMaxN / pfc::kClassesPerBlock);
  c.err_flag = reinterpret_cast<int32_t*>(base + kNaOffErr);
  return pfc::sample_impl(&c, labels, B, r, seed, step, 0xFFFFFFFFu, idx_out, labels_local_out,
                          k_out);
}
