// Score smoothing + per-head top-k (MaskKV Section 3.3: S_keep = argtopk(I, k_{l,h})), and the
// head-level budget formula of Stage 2.
//
// Two stages, because one workgroup per head would leave most of the chip idle:
//   chunk stage  one workgroup per 4096 prompt positions of a head: pools the scores, turns them into
//                order-preserving 32-bit keys, finds the chunk's own top-min(k, chunk) under the same order
//                (larger key first, ties to the lower position) and writes them, in ascending position
//                order, as (key, position) candidates.  Every member of the head's top-k is in its chunk's
//                top-k, so the candidates of all chunks are a superset of the answer, already sorted by
//                position.
//   final stage  one workgroup per head: the same selection over the candidates, emitting positions.
//
// Selection inside a workgroup (16 waves, keys in LDS): the k-th largest key tau is found by range
// refinement: the current key range [lo, hi] is cut into at most 2048 equal bins, an LDS histogram locates
// the bin that holds the k-th largest key, and that bin becomes the new range (three rounds always reach a
// single key).  Scanning everything with LDS atomics is slow when almost every key falls into the same few
// bins (a flat background under a few large scores), so the refinement normally runs on a short candidate
// list: every thread remembers the largest keys among those it handled; the k-th largest of those 1024*c
// remembered keys (c = ceil(k/1024)), or the lower edge of the histogram bin that holds it, is a lower bound
// t0 of tau, because they are a subset of the keys;
// the keys >= t0 - typically little more than k of them - are the candidates.  Inputs with k > 4096, or
// whose candidates do not fit the list, take the whole-array path.
// The kept set is "key > tau" plus the first (k - count_gt) entries with key == tau, emitted in
// ascending order with ballot/popcount prefix sums, each wave walking one contiguous slice.
#include "kernels.hpp"

namespace maskkv {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kChunk = 4096;       // prompt positions per chunk-stage workgroup
constexpr int kSelLdsCap = 32768;  // final stage: keys kept in LDS (128 KB) next to the histogram and the list
constexpr int kBins = 2048;
constexpr int kListCap = 4096;
constexpr int kTopC = 4;           // largest keys remembered per thread

struct SelectParams {
  Lens lens;
  int H, BH, P_max, max_chunks;
  const float* scores;
  int64_t score_stride;
  int window, mode;
  const int32_t* budgets;
  int32_t* idx;
  int32_t* cu;
  int64_t capacity;
  uint32_t* cand_key;  // [BH][max_chunks][kChunk] candidates of the chunk stage
  int32_t* cand_pos;   // [BH][max_chunks][kChunk]
};

__device__ __forceinline__ uint32_t order_key(float v) {
  uint32_t u = __builtin_bit_cast(uint32_t, v);
  if (u == 0x80000000u) u = 0u;                         // -0 and +0 compare equal: one key for both
  return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);  // larger float <=> larger unsigned key
}

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int n = __shfl_up(v, o, 64);
    if (lane >= o) v += n;
  }
  return v;
}

// One histogram vote; lanes of a wave that all vote for the same bin are merged into one atomic.
__device__ __forceinline__ void vote(int* hist, bool cand, uint32_t bin, int lane) {
  const uint64_t cmask = __ballot(cand);
  if (!cmask) return;
  const int leader = __ffsll((unsigned long long)cmask) - 1;
  const uint32_t b0 = __shfl(bin, leader, 64);
  const uint64_t same = __ballot(cand && bin == b0);
  if (same == cmask) {
    if (lane == leader) atomicAdd(&hist[b0], __popcll(cmask));
  } else if (cand) {
    atomicAdd(&hist[bin], 1);
  }
}

// FINAL = false: chunk stage (grid BH x max_chunks).  FINAL = true: final stage (grid BH); LDS_KEYS says
// whether its keys are copied to LDS or read in place from the candidate buffer.  POOL says where the keys come
// from: true = pooled scores (chunk stage), false = the chunk stage's candidates (final stage).  Prompts of at
// most one chunk need no second stage: <FINAL, LDS_KEYS, POOL> = <true, true, true> pools, selects and emits
// positions in one kernel.
template <bool FINAL, bool LDS_KEYS, bool POOL>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelectParams prm) {
  extern __shared__ uint32_t lds_keys[];
  __shared__ int hist[kBins];
  __shared__ uint32_t list[kListCap];
  __shared__ int wsum[kSelWaves][2];
  __shared__ uint32_t wmin[kSelWaves], wmax[kSelWaves];
  __shared__ uint32_t sh_lo, sh_hi;
  __shared__ int sh_krem, sh_base, sh_nlist, sh_bincount;

  const int bh = blockIdx.x;
  const int b = bh / prm.H;
  const int P = prm.lens.P[b];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int kh = min(max(prm.budgets[bh], 0), P);  // the head's budget
  const int nch = (P + kChunk - 1) / kChunk;
  const int kc = min(kh, kChunk);                  // candidates that every full chunk delivers
  const int64_t head_ws = (int64_t)bh * prm.max_chunks * kChunk;

  int base = 0;
  if (FINAL) {
    // ---- offset of this head's slice: exclusive prefix sum of the clamped budgets
    int part = 0;
    for (int i = tid; i < bh; i += kSelThreads) part += min(max(prm.budgets[i], 0), prm.lens.P[i / prm.H]);
    part = wave_incl_scan(part, lane);
    if (lane == 63) wsum[wave][0] = part;
    __syncthreads();
    if (tid == 0) {
      int s = 0;
      for (int w = 0; w < kSelWaves; ++w) s += wsum[w][0];
      sh_base = s;
    }
    __syncthreads();
    base = sh_base;
    if (tid == 0) {
      prm.cu[bh] = base;
      if (bh == prm.BH - 1) prm.cu[prm.BH] = base + kh;
    }
  }
  if (kh == 0) return;

  // ---- the keys of this workgroup: n of them, of which the k largest are wanted
  const int c0 = FINAL ? 0 : (int)blockIdx.y * kChunk;  // chunk stage: first prompt position of the chunk
  if (!FINAL && c0 >= P) return;
  const int n = POOL ? min(kChunk, P - c0) : (nch - 1) * kc + min(kh, P - (nch - 1) * kChunk);
  const int k = FINAL ? kh : min(kh, n);
  // final stage: candidate e of the head sits in chunk min(e / kc, nch-1) of the candidate buffer
  auto cand_slot = [&](int e) -> int64_t {
    const int ch = min(e / kc, nch - 1);
    return head_ws + (int64_t)ch * kChunk + (e - ch * kc);
  };
  auto key_at = [&](int e) -> uint32_t {
    return (FINAL && !LDS_KEYS) ? prm.cand_key[cand_slot(e)] : lds_keys[e];
  };

  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
  uint32_t top[kTopC] = {0u, 0u, 0u, 0u};  // this thread's largest keys, descending (0 = none: below every real key)
  auto remember = [&](uint32_t key) {
    kmin = min(kmin, key);
    kmax = max(kmax, key);
    if (key > top[kTopC - 1]) {
      top[kTopC - 1] = key;
#pragma unroll
      for (int i = kTopC - 1; i > 0; --i) {
        const uint32_t a = top[i - 1], bq = top[i];
        top[i - 1] = max(a, bq);
        top[i] = min(a, bq);
      }
    }
  };
  if (!POOL) {
    for (int e = tid; e < n; e += kSelThreads) {
      const uint32_t key = prm.cand_key[cand_slot(e)];
      if (LDS_KEYS) lds_keys[e] = key;
      remember(key);
    }
  } else {
    // pooled scores -> order-preserving keys
    const float* x = prm.scores + (int64_t)bh * prm.score_stride;
    const int r = (prm.window - 1) / 2;
    if (r <= 3 && prm.mode == MASKKV_POOL_MEAN) {
      // four consecutive positions per thread: ten loads serve four windows of up to seven terms
      for (int e0 = tid * 4; e0 < n; e0 += kSelThreads * 4) {
        const int j0 = c0 + e0;
        float v[10];
#pragma unroll
        for (int i = 0; i < 10; ++i) {
          const int j = j0 - 3 + i;
          v[i] = (j >= 0 && j < P) ? x[j] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = j0 + e;
          if (j < P) {
            const int lo = max(0, j - r), hi = min(P - 1, j + r);
            float acc = 0.f;
            bool first = true;
#pragma unroll
            for (int t = -3; t <= 3; ++t) {
              const int jj = j + t;
              if (jj >= lo && jj <= hi) {  // in-range terms only, lowest index first
                acc = first ? v[e + 3 + t] : __fadd_rn(acc, v[e + 3 + t]);
                first = false;
              }
            }
            const uint32_t key = order_key(__fdiv_rn(acc, (float)(hi - lo + 1)));
            lds_keys[e0 + e] = key;
            remember(key);
          }
        }
      }
    } else {
      for (int e = tid; e < n; e += kSelThreads) {
        const int j = c0 + e;
        const int lo = max(0, j - r);
        const int hi = min(P - 1, j + r);
        float v = x[lo];
        if (prm.mode == MASKKV_POOL_MAX) {
          for (int t = lo + 1; t <= hi; ++t) v = fmaxf(v, x[t]);
        } else {
          for (int t = lo + 1; t <= hi; ++t) v = __fadd_rn(v, x[t]);
          v = __fdiv_rn(v, (float)(hi - lo + 1));
        }
        const uint32_t key = order_key(v);
        lds_keys[e] = key;
        remember(key);
      }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o, 64));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, 64));
  }
  if (lane == 0) {
    wmin[wave] = kmin;
    wmax[wave] = kmax;
  }
  for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0;
  __syncthreads();  // also orders the key writes
  if (tid == 0) {
    uint32_t lo = wmin[0], hi = wmax[0];
    for (int w = 1; w < kSelWaves; ++w) {
      lo = min(lo, wmin[w]);
      hi = max(hi, wmax[w]);
    }
    sh_lo = lo;
    sh_hi = hi;
    sh_krem = k;
    sh_nlist = -1;  // no candidate list yet: rounds scan all n keys
  }
  __syncthreads();

  // ---- range refinement until a single key remains.  State in LDS: the key range [sh_lo, sh_hi], the rank
  // sh_krem wanted inside it, and sh_nlist (>= 0: scan list[0..sh_nlist), < 0: scan all n keys).
  auto refine = [&](int max_rounds) {
    for (int round = 0; round < max_rounds; ++round) {
      const uint32_t lo = sh_lo, hi = sh_hi;
      const int krem = sh_krem;
      const int nlist = sh_nlist;
      if (lo == hi) break;
      const uint32_t width = hi - lo;
      const int shift = max(0, 32 - __clz(width) - 11);  // (width >> shift) < 2048
      const int nb = (int)(width >> shift) + 1;  // (the histogram is all zero here: see the bin walk below)
      if (nlist < 0) {
        for (int e0 = 0; e0 < n; e0 += kSelThreads) {
          const int e = e0 + tid;
          const uint32_t key = e < n ? key_at(e) : 0u;
          const bool cand = e < n && key >= lo && key <= hi;
          vote(hist, cand, cand ? ((key - lo) >> shift) : 0u, lane);
        }
      } else {
        for (int e0 = 0; e0 < nlist; e0 += kSelThreads) {
          const int e = e0 + tid;
          const uint32_t key = e < nlist ? list[e] : 0u;
          const bool cand = e < nlist && key >= lo && key <= hi;
          vote(hist, cand, cand ? ((key - lo) >> shift) : 0u, lane);
        }
      }
      __syncthreads();
      // Walk the bins from the top, two per thread; exactly one bin straddles the krem-th largest key.
      {
        const int b0 = nb - 1 - 2 * tid, b1 = nb - 2 - 2 * tid;
        const int h0 = b0 >= 0 ? hist[b0] : 0;
        const int h1 = b1 >= 0 ? hist[b1] : 0;
        if (b0 >= 0) hist[b0] = 0;  // every bin is read by exactly one thread, which leaves it clean for the
        if (b1 >= 0) hist[b1] = 0;  // next round (at least one barrier away)
        int incl = wave_incl_scan(h0 + h1, lane);
        if (lane == 63) wsum[wave][0] = incl;
        __syncthreads();
        for (int w = 0; w < wave; ++w) incl += wsum[w][0];
        const int before = incl - (h0 + h1);
        if (incl >= krem && before < krem) {
          const bool in0 = before + h0 >= krem;
          const int bsel = in0 ? b0 : b1;
          const int above = in0 ? before : before + h0;
          const uint32_t nlo = lo + ((uint32_t)bsel << shift);
          const uint32_t span = (shift == 0) ? 0u : ((1u << shift) - 1u);
          sh_lo = nlo;
          sh_hi = (uint32_t)min((uint64_t)hi, (uint64_t)nlo + span);
          sh_krem = krem - above;
          sh_bincount = in0 ? h0 : h1;
        }
        __syncthreads();
      }
      // A bin with a single key: that key is the answer, fetch it instead of refining the bin further.
      if (sh_bincount == 1 && sh_lo != sh_hi) {
        const uint32_t nlo = sh_lo, nhi = sh_hi;
        __syncthreads();
        const int cnt = nlist < 0 ? n : nlist;
        for (int e = tid; e < cnt; e += kSelThreads) {
          const uint32_t key = nlist < 0 ? key_at(e) : list[e];
          if (key >= nlo && key <= nhi) {
            sh_lo = key;
            sh_hi = key;
          }
        }
        __syncthreads();
      }
      // First whole-array round: move the chosen bin's keys to the short list if they fit.
      if (nlist < 0 && sh_lo != sh_hi && sh_bincount <= kListCap) {
        const uint32_t nlo = sh_lo, nhi = sh_hi;
        if (tid == 0) sh_nlist = 0;
        __syncthreads();
        for (int e0 = 0; e0 < n; e0 += kSelThreads) {
          const int e = e0 + tid;
          const uint32_t key = e < n ? key_at(e) : 0u;
          const bool cand = e < n && key >= nlo && key <= nhi;
          const uint64_t m = __ballot(cand);
          if (m) {
            int pos = 0;
            if (lane == __ffsll((unsigned long long)m) - 1) pos = atomicAdd(&sh_nlist, __popcll(m));
            pos = __shfl(pos, __ffsll((unsigned long long)m) - 1, 64);
            if (cand) list[pos + __popcll(m & ((1ull << lane) - 1ull))] = key;
          }
        }
        __syncthreads();
      }
    }
  };

  const uint32_t all_lo = sh_lo, all_hi = sh_hi;
  const int c = (k + kSelThreads - 1) / kSelThreads;  // remembered keys per thread that the bound needs
  bool short_list = c <= kTopC;
  if (short_list) {
    // t0 = k-th largest of the remembered keys
    uint32_t tmin = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < kTopC; ++i)
      if (i < c) {
        list[tid * c + i] = top[i];
        tmin = min(tmin, top[i]);
      }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) tmin = min(tmin, (uint32_t)__shfl_xor((int)tmin, o, 64));
    if (lane == 0) wmin[wave] = tmin;
    __syncthreads();
    if (tid == 0) {
      uint32_t lo = wmin[0];
      for (int w = 1; w < kSelWaves; ++w) lo = min(lo, wmin[w]);
      sh_lo = lo;
      sh_hi = all_hi;
      sh_krem = k;
      sh_nlist = kSelThreads * c;
    }
    __syncthreads();
    refine(1);  // one round is enough here: the lower edge of the chosen bin is a lower bound as well
    const uint32_t t0 = sh_lo;
    __syncthreads();  // everyone has read t0 and is done with the remembered keys
    if (tid == 0) sh_nlist = 0;
    __syncthreads();
    for (int e0 = 0; e0 < n; e0 += kSelThreads) {
      const int e = e0 + tid;
      const uint32_t key = e < n ? key_at(e) : 0u;
      const bool cand = e < n && key >= t0;
      const uint64_t m = __ballot(cand);
      if (m) {
        const int leader = __ffsll((unsigned long long)m) - 1;
        int pos = 0;
        if (lane == leader) pos = atomicAdd(&sh_nlist, __popcll(m));
        pos = __shfl(pos, leader, 64) + __popcll(m & ((1ull << lane) - 1ull));
        if (cand && pos < kListCap) list[pos] = key;
      }
    }
    __syncthreads();
    short_list = sh_nlist <= kListCap;
    __syncthreads();
    if (tid == 0) {
      sh_lo = short_list ? t0 : all_lo;
      sh_hi = all_hi;
      sh_krem = k;
      if (!short_list) sh_nlist = -1;
    }
    __syncthreads();
  }
  refine(4);
  const uint32_t tau = sh_lo;
  const int need_eq = sh_krem;  // how many entries equal to tau are kept (lowest first)

  // ---- ordered emit: wave w owns entries [w*seg, (w+1)*seg)
  const int seg = ((n + kSelWaves - 1) / kSelWaves + 63) / 64 * 64;
  const int s0 = wave * seg;
  const int s1 = min(n, s0 + seg);
  int cgt = 0, ceq = 0;
  for (int e0 = s0; e0 < s1; e0 += 64) {
    const int e = e0 + lane;
    const uint32_t kv = e < s1 ? key_at(e) : 0u;
    cgt += __popcll(__ballot(e < s1 && kv > tau));
    ceq += __popcll(__ballot(e < s1 && kv == tau));
  }
  if (lane == 0) {
    wsum[wave][0] = cgt;
    wsum[wave][1] = ceq;
  }
  __syncthreads();
  int gt_before = 0, eq_before = 0;
  for (int w = 0; w < wave; ++w) {
    gt_before += wsum[w][0];
    eq_before += wsum[w][1];
  }
  const int64_t room = prm.capacity - base;  // final stage: rows of idx this head may write
  const int64_t chunk_ws = head_ws + (int64_t)blockIdx.y * kChunk;  // chunk stage: this chunk's candidates
  for (int e0 = s0; e0 < s1; e0 += 64) {
    const int e = e0 + lane;
    const uint32_t kv = e < s1 ? key_at(e) : 0u;
    const bool gt = e < s1 && kv > tau;
    const bool eq = e < s1 && kv == tau;
    const uint64_t mgt = __ballot(gt);
    const uint64_t meq = __ballot(eq);
    const uint64_t below = (1ull << lane) - 1ull;
    const int pg = __popcll(mgt & below);
    const int pe = __popcll(meq & below);
    const int eq_rank = eq_before + pe;
    if (gt || (eq && eq_rank < need_eq)) {
      const int pos = gt_before + pg + min(eq_rank, need_eq);
      if (FINAL) {
        if (pos < room) prm.idx[base + pos] = POOL ? c0 + e : prm.cand_pos[cand_slot(e)];
      } else {
        prm.cand_key[chunk_ws + pos] = kv;
        prm.cand_pos[chunk_ws + pos] = c0 + e;
      }
    }
    gt_before += __popcll(mgt);
    eq_before += __popcll(meq);
  }
}

struct BudgetParams {
  int H, n_query;
  const float* mass;
  int32_t k_l;
  float alpha;
  int32_t* budgets;
};

// k_{l,h} = floor(alpha*k_l + (1-alpha) * N_h * k_l * P_h / sum_j P_j), P_h = mass_h / n_query.
__global__ __launch_bounds__(256) void head_budgets_kernel(const BudgetParams prm) {
  __shared__ float red[256];
  const int b = blockIdx.x;
  float s = 0.f;
  for (int h = threadIdx.x; h < prm.H; h += 256) s += prm.mass[b * prm.H + h] / (float)prm.n_query;
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  const float total = red[0];
  for (int h = threadIdx.x; h < prm.H; h += 256) {
    // a sequence without any prompt mass (empty prompt) has no preference: every head gets k_l
    const float p_hat = total > 0.f ? (prm.mass[b * prm.H + h] / (float)prm.n_query) / total : 1.f / (float)prm.H;
    const float v = prm.alpha * (float)prm.k_l + (1.f - prm.alpha) * (float)prm.H * (float)prm.k_l * p_hat;
    prm.budgets[b * prm.H + h] = (int32_t)floorf(v);
  }
}

bool select_uses_lds(const maskkv_desc* d) { return d->P_max <= kSelLdsCap; }

int64_t select_cand_slots(const maskkv_desc* d) {
  const int64_t max_chunks = (d->P_max + kChunk - 1) / kChunk;
  return (int64_t)d->B * d->H * max_chunks * kChunk;
}

template <typename K>
int raise_lds_limit(K kernel, size_t bytes) {
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) return MASKKV_OK;
  set_error("select: cannot raise dynamic LDS limit: %s", hipGetErrorString(e));
  (void)hipGetLastError();
  return MASKKV_EHIP;
}

}  // namespace

// The (key, position) candidates that the chunk stage hands to the final stage.
size_t select_workspace_bytes(const maskkv_desc* d) {
  return (size_t)select_cand_slots(d) * (sizeof(uint32_t) + sizeof(int32_t));
}

int launch_select(const maskkv_desc* d, const Lens& lens, const float* scores, int64_t score_stride, int window,
                  int mode, const int32_t* budgets, int32_t* idx, int32_t* cu_budget, int64_t capacity,
                  void* workspace, hipStream_t stream) {
  SelectParams prm;
  prm.lens = lens;
  prm.H = d->H;
  prm.BH = d->B * d->H;
  prm.P_max = d->P_max;
  prm.scores = scores;
  prm.score_stride = score_stride;
  prm.window = window;
  prm.mode = mode;
  prm.budgets = budgets;
  prm.idx = idx;
  prm.cu = cu_budget;
  prm.capacity = capacity;
  prm.max_chunks = (d->P_max + kChunk - 1) / kChunk;
  prm.cand_key = reinterpret_cast<uint32_t*>(workspace);
  prm.cand_pos = reinterpret_cast<int32_t*>(prm.cand_key + select_cand_slots(d));
  if (prm.max_chunks == 1) {  // every prompt fits one chunk: pool, select and emit in a single kernel
    hipLaunchKernelGGL((select_kernel<true, true, true>), dim3(prm.BH), dim3(kSelThreads), kChunk * sizeof(uint32_t),
                       stream, prm);
    return check_launch("select (single stage)");
  }
  if (prm.max_chunks > 0) {
    hipLaunchKernelGGL((select_kernel<false, true, true>), dim3(prm.BH, prm.max_chunks), dim3(kSelThreads),
                       kChunk * sizeof(uint32_t), stream, prm);
    if (int e = check_launch("select (chunk stage)")) return e;
  }
  if (select_uses_lds(d)) {
    const size_t dyn = (size_t)((d->P_max + 63) / 64 * 64) * sizeof(uint32_t);
    if (dyn > 48 * 1024) {
      static thread_local bool granted = false;  // one-time opt-in to more than the default dynamic LDS size
      if (!granted) {
        if (int e = raise_lds_limit(&select_kernel<true, true, false>, kSelLdsCap * sizeof(uint32_t))) return e;
        granted = true;
      }
    }
    hipLaunchKernelGGL((select_kernel<true, true, false>), dim3(prm.BH), dim3(kSelThreads), dyn, stream, prm);
  } else {
    hipLaunchKernelGGL((select_kernel<true, false, false>), dim3(prm.BH), dim3(kSelThreads), 0, stream, prm);
  }
  return check_launch("select");
}

int launch_head_budgets(const maskkv_desc* d, const float* prompt_mass, int32_t k_l, float alpha, int32_t* budgets,
                        hipStream_t stream) {
  BudgetParams prm{d->H, d->n_query * query_heads_per_kv(d), prompt_mass, k_l, alpha, budgets};
  hipLaunchKernelGGL(head_budgets_kernel, dim3(d->B), dim3(256), 0, stream, prm);
  return check_launch("head_budgets");
}

}  // namespace maskkv
