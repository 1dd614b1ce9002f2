// Score smoothing + per-head top-k (MaskKV Section 3.3: S_keep = argtopk(I, k_{l,h})), and the head-level
// budget formula of Stage 2.
//
// Two stages, because one workgroup per head would leave most of the chip idle:
//   chunk stage  one workgroup per 4096 prompt positions of a head: pools the scores, turns them into
//                order-preserving 32-bit keys and writes, in ascending position order, every (key, position)
//                whose key is at least t0, the k-th largest key of the chunk (k = the head's budget).  The
//                head's k-th largest key tau is never below a chunk's k-th largest key (fewer than k keys of
//                the whole head are above tau), so every key >= tau of every chunk - all members of the
//                answer and all their ties - is among the candidates.
//   final stage  one workgroup per head: exact selection over the candidates (larger key first, ties to the
//                lower position), positions emitted in ascending order.
// Prompts of at most one chunk skip the chunk stage: the final stage pools the scores itself.
//
// Selection inside a workgroup (both stages): range refinement.  The key range [lo, hi] is cut into at most 2048 equal bins,
// an LDS histogram (votes of a wave for one bin are merged into one atomic) locates the bin that holds the
// k-th largest key, and that bin becomes the range: at most three rounds reach a single key tau.  One wave
// walks the bins (32 consecutive bins per lane, a wave scan, then the owning lane's own 32), so a round is
// two barriers.  The kept set is "key > tau" plus the first (k - count_gt) entries with key == tau, written
// in order with ballot/popcount prefix sums, each wave walking one contiguous slice.
#include "kernels.hpp"

#ifndef SEL_SLACK
#define SEL_SLACK 64
#endif

namespace maskkv {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kChunk = 4096;       // prompt positions per chunk-stage workgroup
constexpr int kSelLdsCap = 32768;  // final stage: keys kept in LDS (128 KB) next to the histogram
constexpr int kBins = 2048;
constexpr int kBinsPerLane = kBins / 64;
constexpr int kHistWords = kBins + kBins / kBinsPerLane;  // one pad word per 32 bins: conflict-free lane walks
constexpr int kChunkSlack = SEL_SLACK;  // a chunk stops refining its threshold at this many keys in the bin
constexpr int kMaxChunks = 1024;   // chunk offsets of a head are kept in LDS: prompts of up to 4 Mi tokens

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
  int lds_words;       // final stage: keys that fit its dynamic LDS
  uint32_t* cand_key;  // [BH][max_chunks][kChunk] candidates of the chunk stage
  int32_t* cand_pos;   // [BH][max_chunks][kChunk]
  int32_t* cand_cnt;   // [BH][max_chunks] candidates per chunk
};

struct SelState {
  uint32_t lo, hi;  // current key range
  int krem;         // rank wanted inside it
  int binpop;       // keys inside it
};

__device__ __forceinline__ uint32_t order_key(float v) {
  uint32_t u = __builtin_bit_cast(uint32_t, v);
  if (u == 0x80000000u) u = 0u;                         // -0 and +0 compare equal: one key for both
  return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);  // larger float <=> larger unsigned key
}

// Wave-level scans and reductions on the data-parallel-primitive path of the vector ALU (row shifts inside the
// rows of 16 lanes, then the two row broadcasts): six dependent vector instructions, no LDS round trips.
template <typename Op>
__device__ __forceinline__ int wave_scan(int v, int identity, Op op) {
  v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x111, 0xf, 0xf, false));  // row_shr:1
  v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x112, 0xf, 0xf, false));  // row_shr:2
  v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x114, 0xf, 0xf, false));  // row_shr:4
  v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x118, 0xf, 0xf, false));  // row_shr:8
  v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x142, 0xa, 0xf, false));  // row_bcast:15 into rows 1, 3
  v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x143, 0xc, 0xf, false));  // row_bcast:31 into rows 2, 3
  return v;
}

__device__ __forceinline__ int wave_incl_scan(int v, int) {
  return wave_scan(v, 0, [](int a, int b) { return a + b; });
}

// Bins are numbered from the top of the range (bin 0 holds the largest keys) and padded by one word per 32.
__device__ __forceinline__ int hist_slot(int top_bin) { return top_bin + top_bin / kBinsPerLane; }

// One histogram vote per lane; the lanes of a wave that vote for the bin of the first (then second) voting
// lane are merged into one atomic each, the rest vote on their own.  Called by all 64 lanes.
__device__ __forceinline__ void vote(int* hist, bool cand, int top_bin, int lane) {
  uint64_t cmask = __ballot(cand);
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    if (!cmask) return;
    const int leader = __ffsll((unsigned long long)cmask) - 1;
    const int b0 = __builtin_amdgcn_readlane(top_bin, leader);
    const bool mine = cand && top_bin == b0;
    const uint64_t same = __ballot(mine);
    if (lane == leader) atomicAdd(&hist[hist_slot(b0)], __popcll(same));
    if (mine) cand = false;
    cmask &= ~same;
  }
  if (cand) atomicAdd(&hist[hist_slot(top_bin)], 1);
}

// Geometry of one refinement round over the key range [lo, hi].
struct Round {
  uint32_t lo;
  int shift, nb;
  __device__ __forceinline__ Round(uint32_t lo_, uint32_t hi_) : lo(lo_) {
    const uint32_t width = hi_ - lo_;
    shift = max(0, 32 - __clz(width) - 11);  // (width >> shift) < 2048
    nb = (int)(width >> shift) + 1;
  }
  __device__ __forceinline__ int top_bin(uint32_t key) const { return nb - 1 - (int)((key - lo) >> shift); }
};

// One wave, after all votes of a round: find the bin (from the top) that holds the krem-th largest key, make it
// the new range, and leave the histogram zeroed for the next round.
__device__ __forceinline__ void pick_bin(int* hist, const Round& rd, uint32_t hi, int krem, int lane, SelState* st) {
  int h[kBinsPerLane];
  int s = 0;
  int* mine = hist + lane * (kBinsPerLane + 1);
#pragma unroll
  for (int j = 0; j < kBinsPerLane; ++j) {
    h[j] = mine[j];
    mine[j] = 0;
    s += h[j];
  }
  const int incl = wave_incl_scan(s, lane);
  int above = incl - s;
  if (incl >= krem && above < krem) {  // exactly one lane owns the bin
    int bsel = -1, pop = 0;
#pragma unroll
    for (int j = 0; j < kBinsPerLane; ++j) {
      if (bsel < 0) {
        if (above + h[j] >= krem) {
          bsel = lane * kBinsPerLane + j;
          pop = h[j];
        } else {
          above += h[j];
        }
      }
    }
    const uint32_t nlo = rd.lo + ((uint32_t)(rd.nb - 1 - bsel) << rd.shift);
    const uint32_t span = rd.shift == 0 ? 0u : ((1u << rd.shift) - 1u);
    st->lo = nlo;
    st->hi = (uint32_t)min((uint64_t)hi, (uint64_t)nlo + span);
    st->krem = krem - above;
    st->binpop = pop;
  }
}

// Pooled score of position j of a head (mean: in-range terms added from the lowest index upwards in fp32, one
// division by their count; max: the maximum), as an order-preserving key.
__device__ __forceinline__ uint32_t pooled_key(const float* x, int j, int P, int r, int mode) {
  const int lo = max(0, j - r);
  const int hi = min(P - 1, j + r);
  float v = x[lo];
  if (mode == MASKKV_POOL_MAX) {
    for (int t = lo + 1; t <= hi; ++t) v = fmaxf(v, x[t]);
  } else {
    for (int t = lo + 1; t <= hi; ++t) v = __fadd_rn(v, x[t]);
    v = __fdiv_rn(v, (float)(hi - lo + 1));
  }
  return order_key(v);
}

// Keys of the four consecutive positions j0 .. j0+3 (0 for positions past the prompt: below every real key).
__device__ __forceinline__ void pooled_keys4(const float* x, int j0, int P, int r, int mode, uint32_t (&key)[4]) {
  if (r <= 3 && mode == MASKKV_POOL_MEAN) {
    // ten loads serve four windows of up to seven terms
    float v[10];
#pragma unroll
    for (int i = 0; i < 10; ++i) {
      const int j = j0 - 3 + i;
      v[i] = (j >= 0 && j < P) ? x[j] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int j = j0 + e;
      key[e] = 0u;
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
        key[e] = order_key(__fdiv_rn(acc, (float)(hi - lo + 1)));
      }
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) key[e] = j0 + e < P ? pooled_key(x, j0 + e, P, r, mode) : 0u;
  }
}

__device__ __forceinline__ uint32_t wave_min(uint32_t v) {
  const int r = wave_scan((int)v, -1, [](int a, int b) { return (int)min((uint32_t)a, (uint32_t)b); });
  return (uint32_t)__builtin_amdgcn_readlane(r, 63);
}
__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
  const int r = wave_scan((int)v, 0, [](int a, int b) { return (int)max((uint32_t)a, (uint32_t)b); });
  return (uint32_t)__builtin_amdgcn_readlane(r, 63);
}

// ---- chunk stage: grid (BH, max_chunks).  Eight waves per SIMD, i.e. at most 64 registers: two of these 1024-thread
// workgroups then fit a compute unit, which halves the rounds a batch with more chunks than compute units needs.
__global__ __launch_bounds__(kSelThreads, 8) void select_chunk_kernel(const SelectParams prm) {
  __shared__ int hist[kHistWords];
  __shared__ uint32_t wmin[kSelWaves], wmax[kSelWaves];
  __shared__ int wsum[kSelWaves];
  __shared__ SelState st;

  const int bh = blockIdx.x;
  const int b = bh / prm.H;
  const int P = prm.lens.P[b];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kh = min(max(prm.budgets[bh], 0), P);
  const int c0 = (int)blockIdx.y * kChunk;
  if (c0 >= P || kh == 0) return;  // the final stage reads neither this chunk's count nor anything of a head without budget
  const int n = min(kChunk, P - c0);
  const int kc = min(kh, n);

  for (int i = tid; i < kHistWords; i += kSelThreads) hist[i] = 0;
  uint32_t key[4];
  pooled_keys4(prm.scores + (int64_t)bh * prm.score_stride, c0 + 4 * tid, P, (prm.window - 1) / 2, prm.mode, key);
  const int nmine = min(max(n - 4 * tid, 0), 4);  // this thread's real keys: key[0 .. nmine)
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (e < nmine) {
      kmin = min(kmin, key[e]);
      kmax = max(kmax, key[e]);
    }
  kmin = wave_min(kmin);
  kmax = wave_max(kmax);
  if (lane == 0) {
    wmin[wave] = kmin;
    wmax[wave] = kmax;
  }
  __syncthreads();
  uint32_t lo = wmin[0], hi = wmax[0];
#pragma unroll
  for (int w = 1; w < kSelWaves; ++w) {
    lo = min(lo, wmin[w]);
    hi = max(hi, wmax[w]);
  }
  // ---- a lower bound of the chunk's kc-th largest key: range refinement over the keys in registers, until the
  // bin that holds it has few keys left (every key of that bin becomes a candidate, so the bound need not be tight;
  // the final stage finds the head's threshold exactly)
  if (kc < n) {
    int krem = kc, binpop = n;
    for (int round = 0; round < 4 && lo != hi && binpop > kChunkSlack; ++round) {
      const Round rd(lo, hi);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool cand = e < nmine && key[e] >= lo && key[e] <= hi;
        vote(hist, cand, cand ? rd.top_bin(key[e]) : 0, lane);
      }
      __syncthreads();
      if (wave == 0) pick_bin(hist, rd, hi, krem, lane, &st);
      __syncthreads();
      lo = st.lo;
      hi = st.hi;
      krem = st.krem;
      binpop = st.binpop;
    }
  }
  const uint32_t t0 = lo;  // kc >= n: the smallest key, everything is a candidate

  // ---- every key >= t0, in position order
  int mine = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) mine += (e < nmine && key[e] >= t0) ? 1 : 0;
  const int incl = wave_incl_scan(mine, lane);
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  int before = incl - mine;
  int total = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int v = wsum[w];
    if (w < wave) before += v;
    total += v;
  }
  const int64_t ws = ((int64_t)bh * prm.max_chunks + blockIdx.y) * kChunk;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    if (e < nmine && key[e] >= t0) {
      prm.cand_key[ws + before] = key[e];
      prm.cand_pos[ws + before] = c0 + 4 * tid + e;
      ++before;
    }
  }
  if (tid == 0) prm.cand_cnt[(int64_t)bh * prm.max_chunks + blockIdx.y] = total;
}

// ---- final stage: grid (BH).  POOL: the keys are the pooled scores of a prompt of at most one chunk;
// otherwise they are the chunk stage's candidates.
template <bool POOL>
__global__ __launch_bounds__(kSelThreads) void select_final_kernel(const SelectParams prm) {
  extern __shared__ uint32_t lds_keys[];
  __shared__ int hist[kHistWords];
  __shared__ int coff[kMaxChunks + 1];  // candidates before chunk c
  __shared__ int wsum[kSelWaves][2];
  __shared__ uint32_t wmin[kSelWaves], wmax[kSelWaves];
  __shared__ SelState st;

  const int bh = blockIdx.x;
  const int b = bh / prm.H;
  const int h = bh - b * prm.H;
  const int P = prm.lens.P[b];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kh = min(max(prm.budgets[bh], 0), P);
  const int nch = POOL ? 1 : (P + kChunk - 1) / kChunk;  // (POOL: the prompt is one flat list)
  const int64_t head_ws = (int64_t)bh * prm.max_chunks * kChunk;

  // ---- offset of this head's slice (exclusive prefix sum of the clamped budgets) and of every chunk's
  // candidates (inclusive scan of the chunk counts): wave scans now, wave totals combined after the barrier
  int part = 0;
  for (int i = tid; i < bh; i += kSelThreads) part += min(max(prm.budgets[i], 0), prm.lens.P[i / prm.H]);
  part = wave_incl_scan(part, lane);
  const int cnt = (!POOL && kh > 0 && tid < nch) ? prm.cand_cnt[(int64_t)bh * prm.max_chunks + tid] : 0;
  const int cincl = wave_incl_scan(cnt, lane);
  if (lane == 63) {
    wsum[wave][0] = part;
    wsum[wave][1] = cincl;
  }
  for (int i = tid; i < kHistWords; i += kSelThreads) hist[i] = 0;
  __syncthreads();
  int base = 0, cbefore = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    base += wsum[w][0];
    if (w < wave) cbefore += wsum[w][1];
  }
  if (tid == 0) {
    prm.cu[bh] = base;
    if (bh == prm.BH - 1) prm.cu[prm.BH] = base + kh;
    coff[0] = 0;
  }
  if (kh == 0) return;
  if (!POOL && tid < nch) coff[tid + 1] = cbefore + cincl;
  __syncthreads();

  const int n = POOL ? P : coff[nch];
  const bool in_lds = n <= prm.lds_words;
  // candidate e of the head sits in chunk c = the last one with coff[c] <= e
  auto slot_of = [&](int e) -> int64_t {
    int a = 0, z = nch;  // coff[a] <= e < coff[z]
    while (z - a > 1) {
      const int m = (a + z) >> 1;
      if (coff[m] <= e)
        a = m;
      else
        z = m;
    }
    return head_ws + (int64_t)a * kChunk + (e - coff[a]);
  };
  auto key_at = [&](int e) -> uint32_t { return in_lds ? lds_keys[e] : prm.cand_key[slot_of(e)]; };

  // ---- the keys (into LDS when they fit) and their range
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
  uint32_t pkey[4] = {0u, 0u, 0u, 0u};  // POOL: this thread's four consecutive keys (n <= 4096)
  if (POOL) {
    pooled_keys4(prm.scores + (int64_t)bh * prm.score_stride, 4 * tid, P, (prm.window - 1) / 2, prm.mode, pkey);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (4 * tid + e < n) {
        lds_keys[4 * tid + e] = pkey[e];
        kmin = min(kmin, pkey[e]);
        kmax = max(kmax, pkey[e]);
      }
  } else {
    // four independent loads in flight per thread (the chunks' candidate lists are read as one flat list)
    for (int e0 = 0; e0 < n; e0 += 4 * kSelThreads) {
      uint32_t kk[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int e = e0 + u * kSelThreads + tid;
        kk[u] = e < n ? prm.cand_key[slot_of(e)] : 0u;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int e = e0 + u * kSelThreads + tid;
        if (e < n) {
          if (in_lds) lds_keys[e] = kk[u];
          kmin = min(kmin, kk[u]);
          kmax = max(kmax, kk[u]);
        }
      }
    }
  }
  kmin = wave_min(kmin);
  kmax = wave_max(kmax);
  if (lane == 0) {
    wmin[wave] = kmin;
    wmax[wave] = kmax;
  }
  __syncthreads();
  uint32_t lo = wmin[0], hi = wmax[0];
#pragma unroll
  for (int w = 1; w < kSelWaves; ++w) {
    lo = min(lo, wmin[w]);
    hi = max(hi, wmax[w]);
  }
  int krem = kh;

  // ---- range refinement until a single key remains (three rounds at most; the bound is only a guard)
  for (int round = 0; round < 4 && lo != hi; ++round) {
    const Round rd(lo, hi);
    for (int e0 = 0; e0 < n; e0 += kSelThreads) {
      const int e = e0 + tid;
      const uint32_t key = e < n ? key_at(e) : 0u;
      const bool cand = e < n && key >= lo && key <= hi;
      vote(hist, cand, cand ? rd.top_bin(key) : 0, lane);
    }
    __syncthreads();
    if (wave == 0) pick_bin(hist, rd, hi, krem, lane, &st);
    __syncthreads();
    lo = st.lo;
    hi = st.hi;
    krem = st.krem;
  }
  const uint32_t tau = lo;
  const int need_eq = krem;  // how many entries equal to tau are kept (lowest positions first)

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
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    if (w < wave) {
      gt_before += wsum[w][0];
      eq_before += wsum[w][1];
    }
  }
  const int64_t room = prm.capacity - base;  // rows of idx this head may write
  const int rows = (int)min((int64_t)kh, max(room, (int64_t)0));
  // The kept candidates' positions sit in global memory.  When there is room behind the keys, the kept entry
  // numbers first go to an LDS list in output order, and the positions are then fetched with independent loads
  // (one per thread) instead of one dependent load per step of a wave's slice.
  const bool listed = !POOL && in_lds && n + kh <= prm.lds_words;
  uint32_t* kept = lds_keys + n;
  for (int e0 = s0; e0 < s1; e0 += 64) {
    const int e = e0 + lane;
    const uint32_t kv = e < s1 ? key_at(e) : 0u;
    const bool gt = e < s1 && kv > tau;
    const bool eq = e < s1 && kv == tau;
    const uint64_t mgt = __ballot(gt);
    const uint64_t meq = __ballot(eq);
    const uint64_t below = (1ull << lane) - 1ull;
    const int eq_rank = eq_before + __popcll(meq & below);
    if (gt || (eq && eq_rank < need_eq)) {
      const int pos = gt_before + __popcll(mgt & below) + min(eq_rank, need_eq);
      if (pos < rows) {
        if (POOL)
          prm.idx[base + pos] = e;
        else if (listed)
          kept[pos] = (uint32_t)e;
        else
          prm.idx[base + pos] = prm.cand_pos[slot_of(e)];
      }
    }
    gt_before += __popcll(mgt);
    eq_before += __popcll(meq);
  }
  if (listed) {
    __syncthreads();
    for (int rr = tid; rr < rows; rr += kSelThreads) {
      const int pos = prm.cand_pos[slot_of((int)kept[rr])];
      prm.idx[base + rr] = pos;
    }
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

int64_t select_chunks(const maskkv_desc* d) { return ((int64_t)d->P_max + kChunk - 1) / kChunk; }

int64_t select_cand_slots(const maskkv_desc* d) { return (int64_t)d->B * d->H * select_chunks(d) * kChunk; }

size_t select_count_bytes(const maskkv_desc* d) {
  return ((size_t)((int64_t)d->B * d->H * select_chunks(d)) * sizeof(int32_t) + 255) / 256 * 256;
}

}  // namespace

// Longest prompt the final stage can index (its chunk offsets live in LDS).
int64_t select_max_prompt() { return (int64_t)kMaxChunks * kChunk; }

// The (key, position) candidates that the chunk stage hands to the final stage, and their count per chunk.
size_t select_workspace_bytes(const maskkv_desc* d) {
  if (select_chunks(d) <= 1) return 0;  // single-chunk prompts are selected in one kernel
  return (size_t)select_cand_slots(d) * (sizeof(uint32_t) + sizeof(int32_t)) + select_count_bytes(d);
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
  prm.max_chunks = (int)select_chunks(d);
  prm.cand_key = reinterpret_cast<uint32_t*>(workspace);
  prm.cand_pos = reinterpret_cast<int32_t*>(prm.cand_key + select_cand_slots(d));
  prm.cand_cnt = prm.cand_pos + select_cand_slots(d);
  prm.lds_words = (int)min((int64_t)kSelLdsCap, ((int64_t)max(d->P_max, 1) + 63) / 64 * 64);
  const size_t dyn = (size_t)prm.lds_words * sizeof(uint32_t);
  static bool granted = false;  // one-time opt-in to more than the default dynamic LDS size
  if (!granted) {
    const size_t want = (size_t)kSelLdsCap * sizeof(uint32_t);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_final_kernel<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)want);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_final_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)want);
    if (e != hipSuccess) {
      set_error("select: cannot raise dynamic LDS limit: %s", hipGetErrorString(e));
      (void)hipGetLastError();
      return MASKKV_EHIP;
    }
    granted = true;
  }
  if (prm.max_chunks <= 1) {  // every prompt fits one chunk: pool, select and emit in a single kernel
    hipLaunchKernelGGL((select_final_kernel<true>), dim3(prm.BH), dim3(kSelThreads), dyn, stream, prm);
    return check_launch("select (single stage)");
  }
  hipLaunchKernelGGL(select_chunk_kernel, dim3(prm.BH, prm.max_chunks), dim3(kSelThreads), 0, stream, prm);
  if (int e = check_launch("select (chunk stage)")) return e;
  hipLaunchKernelGGL((select_final_kernel<false>), dim3(prm.BH), dim3(kSelThreads), dyn, stream, prm);
  return check_launch("select (final stage)");
}

int launch_head_budgets(const maskkv_desc* d, const float* prompt_mass, int32_t k_l, float alpha, int32_t* budgets,
                        hipStream_t stream) {
  BudgetParams prm{d->H, d->n_query * query_heads_per_kv(d), prompt_mass, k_l, alpha, budgets};
  hipLaunchKernelGGL(head_budgets_kernel, dim3(d->B), dim3(256), 0, stream, prm);
  return check_launch("head_budgets");
}

}  // namespace maskkv
