// Score smoothing + per-head top-k (MaskKV Section 3.3: S_keep = argtopk(I, k_{l,h})), and the
// head-level budget formula of Stage 2.
//
// One workgroup of 16 waves serves one (b, h).  The pooled scores are turned into order-preserving
// 32-bit keys and kept in LDS (or in a global scratch row when the prompt is longer than LDS holds).
// The k-th largest key tau is found by an MSB-first radix select with 8-bit digits (LDS histogram,
// wave-aggregated atomics when a wave's digits agree); the kept set is then "key > tau" plus the first
// (k - count_gt) positions with key == tau, emitted in ascending position order with ballot/popcount
// prefix sums, each wave walking one contiguous slice of the prompt.
#include "kernels.hpp"

namespace maskkv {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelLdsCap = 36864;  // keys that fit the 160 KB LDS next to the small arrays (144 KB)

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

template <bool LDS_KEYS>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelectParams prm) {
  extern __shared__ uint32_t lds_keys[];
  __shared__ int hist[256];
  __shared__ int wsum[kSelWaves][2];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_krem;
  __shared__ int sh_base;

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

  // ---- pooled scores -> order-preserving keys
  const float* x = prm.scores + (int64_t)bh * prm.score_stride;
  const int r = (prm.window - 1) / 2;
  for (int j = tid; j < P; j += kSelThreads) {
    const int lo = max(0, j - r);
    const int hi = min(P - 1, j + r);
    float v;
    if (prm.mode == MASKKV_POOL_MAX) {
      v = x[lo];
      for (int t = lo + 1; t <= hi; ++t) v = fmaxf(v, x[t]);
    } else {
      v = x[lo];
      for (int t = lo + 1; t <= hi; ++t) v = __fadd_rn(v, x[t]);
      v = __fdiv_rn(v, (float)(hi - lo + 1));
    }
    keys[j] = order_key(v);
  }
  if (tid == 0) {
    sh_prefix = 0u;
    sh_krem = k;
  }

  // ---- radix select of the k-th largest key
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();  // also orders the key writes (and the global scratch writes within the block)
    const uint32_t prefix = sh_prefix;
    const int krem = sh_krem;
    const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
    for (int j0 = 0; j0 < P; j0 += kSelThreads) {
      const int j = j0 + tid;
      const bool cand = j < P && ((keys[j] & himask) == prefix);
      const uint32_t digit = cand ? ((keys[j] >> shift) & 255u) : 0u;
      const uint64_t cmask = __ballot(cand);
      if (cmask) {
        const int leader = __ffsll((unsigned long long)cmask) - 1;
        const uint32_t d0 = __shfl(digit, leader, 64);
        const uint64_t same = __ballot(cand && digit == d0);
        if (same == cmask) {
          if (lane == leader) atomicAdd(&hist[d0], __popcll(cmask));
        } else if (cand) {
          atomicAdd(&hist[digit], 1);
        }
      }
    }
    __syncthreads();
    // suffix counts from the top bin; exactly one bin straddles the k-th largest
    // (waves 0..3 hold the 256 bins, top bin first)
    int val = 0, incl = 0;
    if (tid < 256) {
      val = hist[255 - tid];
      incl = wave_incl_scan(val, lane);
      if (lane == 63) wsum[wave][0] = incl;
    }
    __syncthreads();
    if (tid < 256) {
      for (int w = 0; w < wave; ++w) incl += wsum[w][0];
      if (incl >= krem && incl - val < krem) {
        sh_prefix = prefix | ((uint32_t)(255 - tid) << shift);
        sh_krem = krem - (incl - val);
      }
    }
    __syncthreads();
  }
  const uint32_t tau = sh_prefix;
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
