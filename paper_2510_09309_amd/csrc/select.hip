// Score smoothing + per-head top-k (MaskKV Section 3.3: S_keep = argtopk(I, k_{l,h})), and the
// head-level budget formula of Stage 2.
//
// One workgroup of 16 waves serves one (b, h).  The pooled scores are turned into order-preserving
// 32-bit keys and kept in LDS (or in a global scratch row when the prompt is longer than LDS holds).
// The k-th largest key tau is found by range refinement: the current key range [lo, hi] (initially the
// minimum and maximum key of the head) is cut into at most 2048 equal bins, an LDS histogram locates the
// bin that holds the k-th largest key, and that bin becomes the new range.  Because the bins follow the
// data's own range the histogram stays spread out (few colliding LDS atomics) for the narrow score
// distributions attention produces, and three rounds always reach a single key.  After the first round
// the candidates of the chosen bin are copied to a short LDS list, so later rounds touch only those.
// The kept set is "key > tau" plus the first (k - count_gt) positions with key == tau, emitted in
// ascending position order with ballot/popcount prefix sums, each wave walking one contiguous slice.
#include "kernels.hpp"

namespace maskkv {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelLdsCap = 32768;  // keys kept in LDS (128 KB) next to the histogram and the candidate list
constexpr int kBins = 2048;
constexpr int kListCap = 2048;

struct SelectParams {
  Lens lens;
  int H, BH, P_max;
  const float* scores;
  int64_t score_stride;
  int window, mode;
  const int32_t* budgets;
  int32_t* idx;
  int32_t* cu;
  int64_t capacity;
  uint32_t* gkeys;  // [BH][P_max] scratch when the keys do not fit LDS
};

__device__ __forceinline__ uint32_t order_key(float v) {
  const uint32_t u = __builtin_bit_cast(uint32_t, v);
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

template <bool LDS_KEYS>
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
  uint32_t* keys = LDS_KEYS ? lds_keys : (prm.gkeys + (int64_t)bh * prm.P_max);

  // ---- offset of this head's slice: exclusive prefix sum of the clamped budgets
  {
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
  }
  const int base = sh_base;
  const int k = min(max(prm.budgets[bh], 0), P);
  if (tid == 0) {
    prm.cu[bh] = base;
    if (bh == prm.BH - 1) prm.cu[prm.BH] = base + k;
  }
  if (k == 0) return;

  // ---- pooled scores -> order-preserving keys, and the key range of the head
  const float* x = prm.scores + (int64_t)bh * prm.score_stride;
  const int r = (prm.window - 1) / 2;
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
  if (r <= 3 && prm.mode == MASKKV_POOL_MEAN) {
    // four consecutive positions per thread: ten loads serve four windows of up to seven terms
    for (int j0 = tid * 4; j0 < P; j0 += kSelThreads * 4) {
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
          keys[j] = key;
          kmin = min(kmin, key);
          kmax = max(kmax, key);
        }
      }
    }
  } else {
    for (int j = tid; j < P; j += kSelThreads) {
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
      keys[j] = key;
      kmin = min(kmin, key);
      kmax = max(kmax, key);
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
  __syncthreads();  // also orders the key writes (and the global scratch writes within the block)
  if (tid == 0) {
    uint32_t lo = wmin[0], hi = wmax[0];
    for (int w = 1; w < kSelWaves; ++w) {
      lo = min(lo, wmin[w]);
      hi = max(hi, wmax[w]);
    }
    sh_lo = lo;
    sh_hi = hi;
    sh_krem = k;
    sh_nlist = -1;  // no candidate list yet: rounds scan the whole head
  }
  __syncthreads();

  // ---- range refinement until a single key remains
  for (int round = 0; round < 4; ++round) {
    const uint32_t lo = sh_lo, hi = sh_hi;
    const int krem = sh_krem;
    const int nlist = sh_nlist;
    if (lo == hi) break;
    const uint32_t width = hi - lo;
    const int shift = max(0, 32 - __clz(width) - 11);  // (width >> shift) < 2048
    const int nb = (int)(width >> shift) + 1;
    for (int i = tid; i < nb; i += kSelThreads) hist[i] = 0;
    __syncthreads();
    if (nlist < 0) {
      for (int j0 = 0; j0 < P; j0 += kSelThreads) {
        const int j = j0 + tid;
        const uint32_t key = j < P ? keys[j] : 0u;
        const bool cand = j < P && key >= lo && key <= hi;
        vote(hist, cand, cand ? ((key - lo) >> shift) : 0u, lane);
      }
    } else {
      for (int j0 = 0; j0 < nlist; j0 += kSelThreads) {
        const int j = j0 + tid;
        const uint32_t key = j < nlist ? list[j] : 0u;
        const bool cand = j < nlist && key >= lo && key <= hi;
        vote(hist, cand, cand ? ((key - lo) >> shift) : 0u, lane);
      }
    }
    __syncthreads();
    // Walk the bins from the top, two per thread; exactly one bin straddles the krem-th largest key.
    {
      const int b0 = nb - 1 - 2 * tid, b1 = nb - 2 - 2 * tid;
      const int h0 = b0 >= 0 ? hist[b0] : 0;
      const int h1 = b1 >= 0 ? hist[b1] : 0;
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
    // First round: move the chosen bin's candidates to the short list if they fit.
    if (nlist < 0 && sh_lo != sh_hi && sh_bincount <= kListCap) {
      const uint32_t nlo = sh_lo, nhi = sh_hi;
      if (tid == 0) sh_nlist = 0;
      __syncthreads();
      for (int j0 = 0; j0 < P; j0 += kSelThreads) {
        const int j = j0 + tid;
        const uint32_t key = j < P ? keys[j] : 0u;
        const bool cand = j < P && key >= nlo && key <= nhi;
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
  const uint32_t tau = sh_lo;
  const int need_eq = sh_krem;  // how many positions equal to tau are kept (lowest positions first)

  // ---- ordered emit: wave w owns positions [w*seg, (w+1)*seg)
  const int seg = ((P + kSelWaves - 1) / kSelWaves + 63) / 64 * 64;
  const int s0 = wave * seg;
  const int s1 = min(P, s0 + seg);
  int cgt = 0, ceq = 0;
  for (int j0 = s0; j0 < s1; j0 += 64) {
    const int j = j0 + lane;
    const uint32_t kv = j < s1 ? keys[j] : 0u;
    cgt += __popcll(__ballot(j < s1 && kv > tau));
    ceq += __popcll(__ballot(j < s1 && kv == tau));
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
  int32_t* out = prm.idx + base;
  const int64_t room = prm.capacity - base;  // rows of idx this head may write
  for (int j0 = s0; j0 < s1; j0 += 64) {
    const int j = j0 + lane;
    const uint32_t kv = j < s1 ? keys[j] : 0u;
    const bool gt = j < s1 && kv > tau;
    const bool eq = j < s1 && kv == tau;
    const uint64_t mgt = __ballot(gt);
    const uint64_t meq = __ballot(eq);
    const uint64_t below = (1ull << lane) - 1ull;
    const int pg = __popcll(mgt & below);
    const int pe = __popcll(meq & below);
    const int eq_rank = eq_before + pe;
    if (gt || (eq && eq_rank < need_eq)) {
      const int pos = gt_before + pg + min(eq_rank, need_eq);
      if (pos < room) out[pos] = j;
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
    const float p_hat = (prm.mass[b * prm.H + h] / (float)prm.n_query) / total;
    const float v = prm.alpha * (float)prm.k_l + (1.f - prm.alpha) * (float)prm.H * (float)prm.k_l * p_hat;
    prm.budgets[b * prm.H + h] = (int32_t)floorf(v);
  }
}

bool select_uses_lds(const maskkv_desc* d) { return d->P_max <= kSelLdsCap; }

}  // namespace

size_t select_workspace_bytes(const maskkv_desc* d) {
  if (select_uses_lds(d)) return 0;
  return (size_t)d->B * d->H * (size_t)d->P_max * sizeof(uint32_t);
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
  prm.gkeys = reinterpret_cast<uint32_t*>(workspace);
  const dim3 grid(prm.BH), block(kSelThreads);
  if (select_uses_lds(d)) {
    const size_t dyn = (size_t)((d->P_max + 63) / 64 * 64) * sizeof(uint32_t);
    if (dyn > 48 * 1024) {
      // one-time opt-in to more than the default dynamic LDS size
      static thread_local size_t granted = 0;
      if (dyn > granted) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel<true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kSelLdsCap * 4));
        if (e != hipSuccess) {
          set_error("select: cannot raise dynamic LDS limit: %s", hipGetErrorString(e));
          (void)hipGetLastError();
          return MASKKV_EHIP;
        }
        granted = kSelLdsCap * 4;
      }
    }
    hipLaunchKernelGGL(select_kernel<true>, grid, block, dyn, stream, prm);
  } else {
    hipLaunchKernelGGL(select_kernel<false>, grid, block, 0, stream, prm);
  }
  return check_launch("select");
}

int launch_head_budgets(const maskkv_desc* d, const float* prompt_mass, int32_t k_l, float alpha, int32_t* budgets,
                        hipStream_t stream) {
  BudgetParams prm{d->H, d->n_query, prompt_mass, k_l, alpha, budgets};
  hipLaunchKernelGGL(head_budgets_kernel, dim3(d->B), dim3(256), 0, stream, prm);
  return check_launch("head_budgets");
}

}  // namespace maskkv
