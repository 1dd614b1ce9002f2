// Mask-Voting scoring kernels (MaskKV Section 3.3, Stage 1):
//   A = softmax_row(Q_mask K_full^T * scale),  I_j = sum_i A_ij over the prompt columns.
//
// A column sum needs every row's final softmax normaliser, so the logits are formed twice:
//   pass 1  row statistics (running max and sum of exponentials, base 2) per key chunk,
//   merge   per-row log-sum-exp over the chunks (+ the prompt's share of each row = prompt mass),
//   pass 2  logits again, p = exp2(s*c - lse), summed over the queries for every prompt key.
// Storing the n_m x N logits instead would cost far more HBM traffic than the second MFMA pass.
//
// Tiling: one workgroup = 4 waves = one key chunk of one (b, h).  Each wave keeps 64 queries as MFMA
// operands in registers; 64-key tiles of K stream through a padded, double-buffered LDS tile shared by
// the four waves.  Pass 1 puts keys on the MFMA row axis so that a lane owns one query and the softmax
// statistics never leave the lane; pass 2 puts queries on the row axis so that the sum over queries is
// in-lane adds plus one cross-lane exchange.
#include "kernels.hpp"

namespace maskkv {

namespace {

constexpr int kScoreThreads = 256;
constexpr int kScoreWaves = 4;
constexpr int kQPerWave = 64;                          // two 32-row MFMA blocks
constexpr int kQPerGroup = kScoreWaves * kQPerWave;    // queries covered per sweep of the chunk

template <typename T, int D>
struct ScoreCfg {
  static constexpr int kRowB = D * (int)sizeof(T);     // bytes per K row
  static constexpr int kRowP = kRowB + 16;             // padded LDS row: conflict-free 16-byte reads
  static constexpr int kSteps = kRowB / 32;            // fragments per row
  static constexpr int kTK = (kRowB <= 256) ? 64 : 32; // keys per tile
  static constexpr int kPieces = kTK * kRowB / 16 / kScoreThreads;  // 16-byte pieces per thread per tile
  static constexpr int kPiecesPerRow = kRowB / 16;
};

struct ScoreParams {
  View Q, K;
  Lens lens;
  int H, n_resp, n_query;
  int chunk;          // keys per chunk (multiple of the tile)
  int nch_max;        // chunk slots per (b, h) in the statistics buffer
  float c;            // scale * log2(e)
  float2* stats;      // [B*H][nch_max][n_query] (max, sum) in the base-2 domain
  float* lse2;        // [B*H][n_query]
  float* scores;      // [B*H][score_stride]
  int64_t score_stride;
  float* prompt_mass; // [B*H] or null
};

// Key range of chunk slot `ch` for a sequence with P prompt keys: prompt chunks first, then response chunks.
// Chunks never straddle the prompt/response boundary.  Returns false for an unused slot.
__device__ __forceinline__ bool chunk_range(int ch, int P, int n_resp, int chunk, int& k0, int& k1, bool& is_prompt) {
  const int npc = (P + chunk - 1) / chunk;
  const int nrc = (n_resp + chunk - 1) / chunk;
  if (ch < npc) {
    k0 = ch * chunk;
    k1 = min(P, k0 + chunk);
    is_prompt = true;
    return true;
  }
  const int rc = ch - npc;
  if (rc < nrc) {
    k0 = P + rc * chunk;
    k1 = min(P + n_resp, k0 + chunk);
    is_prompt = false;
    return true;
  }
  return false;
}

template <typename T, int D>
__device__ __forceinline__ void load_tile_global(const View& K, int b, int h, int key0, int klast, u32x4 (&regs)[ScoreCfg<T, D>::kPieces]) {
  using C = ScoreCfg<T, D>;
#pragma unroll
  for (int i = 0; i < C::kPieces; ++i) {
    const int p = threadIdx.x + i * kScoreThreads;
    const int row = p / C::kPiecesPerRow;
    const int col = p % C::kPiecesPerRow;
    const int key = min(key0 + row, klast);  // rows past the chunk end re-read the last valid row
    regs[i] = *reinterpret_cast<const u32x4*>(K.row(b, h, key) + col * 16);
  }
}

template <typename T, int D>
__device__ __forceinline__ void store_tile_lds(char* buf, const u32x4 (&regs)[ScoreCfg<T, D>::kPieces]) {
  using C = ScoreCfg<T, D>;
#pragma unroll
  for (int i = 0; i < C::kPieces; ++i) {
    const int p = threadIdx.x + i * kScoreThreads;
    const int row = p / C::kPiecesPerRow;
    const int col = p % C::kPiecesPerRow;
    *reinterpret_cast<u32x4*>(buf + row * C::kRowP + col * 16) = regs[i];
  }
}

// PASS 1: row statistics.  PASS 2: column sums.
template <typename T, int D, int PASS>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(const ScoreParams prm) {
  using C = ScoreCfg<T, D>;
  __shared__ __attribute__((aligned(16))) char kt[2][C::kTK * C::kRowP];
  extern __shared__ __attribute__((aligned(16))) float colsum[];  // pass 2: [kScoreWaves][chunk]

  const int bh = blockIdx.y;
  const int b = bh / prm.H;
  const int h = bh % prm.H;
  const int P = prm.lens.P[b];
  int k0, k1;
  bool is_prompt;
  if (!chunk_range(blockIdx.x, P, prm.n_resp, prm.chunk, k0, k1, is_prompt)) return;
  if (PASS == 2 && !is_prompt) return;

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int r = lane & 31;
  const int g = lane >> 5;
  const int ntiles = (k1 - k0 + C::kTK - 1) / C::kTK;
  const float c = prm.c;

  for (int qg = 0; qg < prm.n_query; qg += kQPerGroup) {
    const int q0 = qg + wave * kQPerWave;
    // Query fragments stay in registers for the whole chunk.
    u32x4 qf[2][C::kSteps];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int q = q0 + blk * 32 + r;
#pragma unroll
      for (int ks = 0; ks < C::kSteps; ++ks) {
        if (q < prm.n_query)
          qf[blk][ks] = *reinterpret_cast<const u32x4*>(prm.Q.row(b, h, q) + ks * 32 + g * 16);
        else
          qf[blk][ks] = u32x4{0u, 0u, 0u, 0u};
      }
    }

    // pass 1 state: this lane's running (max, sum) for query q0 + 32*blk + r over the keys it sees
    float run_m[2] = {kNegBig, kNegBig};
    float run_l[2] = {0.f, 0.f};
    // pass 2 state: -lse2 of the 16 query rows this lane sees in each block
    float nb[2][16];
    if (PASS == 2) {
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int q = q0 + blk * 32 + 8 * (i / 4) + 4 * g + (i % 4);
          nb[blk][i] = (q < prm.n_query) ? -prm.lse2[(int64_t)bh * prm.n_query + q] : -INFINITY;
        }
    }

    u32x4 stage[C::kPieces];
    __syncthreads();  // previous sweep's readers are done with the tile buffers
    load_tile_global<T, D>(prm.K, b, h, k0, k1 - 1, stage);
    store_tile_lds<T, D>(kt[0], stage);
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
      const int key0 = k0 + t * C::kTK;
      if (t + 1 < ntiles) load_tile_global<T, D>(prm.K, b, h, key0 + C::kTK, k1 - 1, stage);
      const char* buf = kt[t & 1];

#pragma unroll
      for (int kb = 0; kb < C::kTK / 32; ++kb) {
        f32x16 acc0 = {}, acc1 = {};
#pragma unroll
        for (int ks = 0; ks < C::kSteps; ++ks) {
          const u32x4 kf = *reinterpret_cast<const u32x4*>(buf + (kb * 32 + r) * C::kRowP + ks * 32 + g * 16);
          if (PASS == 1) {  // S^T block: keys on rows, queries on columns
            mfma_step<T>(kf, qf[0][ks], acc0);
            mfma_step<T>(kf, qf[1][ks], acc1);
          } else {          // S block: queries on rows, keys on columns
            mfma_step<T>(qf[0][ks], kf, acc0);
            mfma_step<T>(qf[1][ks], kf, acc1);
          }
        }
        if (PASS == 1) {
          const int nvalid = k1 - (key0 + kb * 32);  // rows >= nvalid of this block are past the chunk end
          if (nvalid < 32) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int row = 8 * (i / 4) + 4 * g + (i % 4);
              if (row >= nvalid) {
                acc0[i] = -INFINITY;
                acc1[i] = -INFINITY;
              }
            }
          }
#pragma unroll
          for (int blk = 0; blk < 2; ++blk) {
            const f32x16& a = blk ? acc1 : acc0;
            float bm = a[0];
#pragma unroll
            for (int i = 1; i < 16; ++i) bm = fmaxf(bm, a[i]);
            const float m_new = fmaxf(run_m[blk], bm * c);
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) s += fast_exp2(fmaf(a[i], c, -m_new));
            run_l[blk] = run_l[blk] * fast_exp2(run_m[blk] - m_new) + s;
            run_m[blk] = m_new;
          }
        } else {
          float cs = 0.f;
#pragma unroll
          for (int i = 0; i < 16; ++i) cs += fast_exp2(fmaf(acc0[i], c, nb[0][i]));
#pragma unroll
          for (int i = 0; i < 16; ++i) cs += fast_exp2(fmaf(acc1[i], c, nb[1][i]));
          cs += xor32(cs);
          if (g == 0) {
            float* dst = colsum + wave * prm.chunk + (key0 - k0) + kb * 32 + r;
            *dst = (qg == 0) ? cs : (*dst + cs);
          }
        }
      }

      if (t + 1 < ntiles) store_tile_lds<T, D>(kt[(t + 1) & 1], stage);
      __syncthreads();
    }

    if (PASS == 1) {
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) {
        const float m_o = xor32(run_m[blk]);
        const float l_o = xor32(run_l[blk]);
        const float m = fmaxf(run_m[blk], m_o);
        const float l = run_l[blk] * fast_exp2(run_m[blk] - m) + l_o * fast_exp2(m_o - m);
        const int q = q0 + blk * 32 + r;
        if (g == 0 && q < prm.n_query)
          prm.stats[((int64_t)bh * prm.nch_max + blockIdx.x) * prm.n_query + q] = make_float2(m, l);
      }
    }
  }

  if (PASS == 2) {
    // colsum was last written before the final barrier of the tile loop
    float* out = prm.scores + (int64_t)bh * prm.score_stride + k0;
    for (int j = threadIdx.x; j < k1 - k0; j += kScoreThreads) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < kScoreWaves; ++w) s += colsum[w * prm.chunk + j];
      out[j] = s;
    }
  }
}

// Merge the per-chunk statistics of every query row into its base-2 log-sum-exp; the prompt chunks'
// share of each row's normaliser, summed over the rows, is the mask-to-prompt attention mass.
__global__ __launch_bounds__(256) void score_merge_kernel(const ScoreParams prm) {
  __shared__ float red[256];
  const int bh = blockIdx.x;
  const int b = bh / prm.H;
  const int P = prm.lens.P[b];
  const int npc = (P + prm.chunk - 1) / prm.chunk;
  const int nch = npc + (prm.n_resp + prm.chunk - 1) / prm.chunk;
  float mass = 0.f;
  for (int q = threadIdx.x; q < prm.n_query; q += 256) {
    const float2* st = prm.stats + (int64_t)bh * prm.nch_max * prm.n_query + q;
    float M = kNegBig;
    for (int ch = 0; ch < nch; ++ch) M = fmaxf(M, st[(int64_t)ch * prm.n_query].x);
    float L = 0.f, Lp = 0.f;
    for (int ch = 0; ch < nch; ++ch) {
      const float2 v = st[(int64_t)ch * prm.n_query];
      const float w = v.y * fast_exp2(v.x - M);
      L += w;
      if (ch < npc) Lp += w;
    }
    prm.lse2[(int64_t)bh * prm.n_query + q] = M + __log2f(L);
    mass += Lp / L;
  }
  red[threadIdx.x] = mass;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0 && prm.prompt_mass) prm.prompt_mass[bh] = red[0];
}

int score_chunk_keys(const maskkv_desc* d) {
  // Aim at roughly four workgroups per compute unit, chunks of 256..1024 keys.
  const int64_t total = (int64_t)d->B * d->H * ((int64_t)d->P_max + d->n_resp);
  int64_t c = (total + 1023) / 1024;
  c = (c + 63) / 64 * 64;
  if (c < 256) c = 256;
  if (c > 1024) c = 1024;
  return (int)c;
}

int mark(void* const* events, int i, hipStream_t stream) {
  if (!events || !events[i]) return MASKKV_OK;
  const hipError_t e = hipEventRecord(reinterpret_cast<hipEvent_t>(events[i]), stream);
  if (e == hipSuccess) return MASKKV_OK;
  set_error("score: hipEventRecord(events[%d]): %s", i, hipGetErrorString(e));
  return MASKKV_EHIP;
}

template <typename T, int D>
int launch_score_t(const ScoreParams& prm, int B, hipStream_t stream, void* const* events) {
  const dim3 block(kScoreThreads);
  const dim3 grid1(prm.nch_max, B * prm.H);
  if (int e = mark(events, 0, stream)) return e;
  hipLaunchKernelGGL((score_kernel<T, D, 1>), grid1, block, 0, stream, prm);
  if (int e = check_launch("score pass 1")) return e;
  if (int e = mark(events, 1, stream)) return e;
  hipLaunchKernelGGL(score_merge_kernel, dim3(B * prm.H), dim3(256), 0, stream, prm);
  if (int e = check_launch("score merge")) return e;
  if (int e = mark(events, 2, stream)) return e;
  int npc_max = 0;
  for (int b = 0; b < B; ++b) npc_max = max(npc_max, (prm.lens.P[b] + prm.chunk - 1) / prm.chunk);
  if (npc_max > 0) {
    const dim3 grid2(npc_max, B * prm.H);
    const size_t dyn = sizeof(float) * kScoreWaves * prm.chunk;
    hipLaunchKernelGGL((score_kernel<T, D, 2>), grid2, block, dyn, stream, prm);
    if (int e = check_launch("score pass 2")) return e;
  }
  return mark(events, 3, stream);
}

}  // namespace

size_t score_workspace_bytes(const maskkv_desc* d) {
  const int chunk = score_chunk_keys(d);
  const int64_t nch = (d->P_max + chunk - 1) / chunk + (d->n_resp + chunk - 1) / chunk;
  const int64_t bh = (int64_t)d->B * d->H;
  size_t stats = (size_t)(bh * nch * d->n_query) * sizeof(float2);
  stats = (stats + 255) / 256 * 256;
  const size_t lse = (size_t)(bh * d->n_query) * sizeof(float);
  return stats + (lse + 255) / 256 * 256;
}

int launch_score(const maskkv_desc* d, const View& Q, const View& K, const Lens& lens, float scale, float* scores,
                 int64_t score_stride, float* prompt_mass, void* workspace, hipStream_t stream,
                 void* const* events) {
  ScoreParams prm;
  prm.Q = Q;
  prm.K = K;
  prm.lens = lens;
  prm.H = d->H;
  prm.n_resp = d->n_resp;
  prm.n_query = d->n_query;
  prm.chunk = score_chunk_keys(d);
  prm.nch_max = (d->P_max + prm.chunk - 1) / prm.chunk + (d->n_resp + prm.chunk - 1) / prm.chunk;
  prm.c = scale * kLog2e;
  const int64_t bh = (int64_t)d->B * d->H;
  size_t stats = (size_t)(bh * prm.nch_max * d->n_query) * sizeof(float2);
  stats = (stats + 255) / 256 * 256;
  prm.stats = reinterpret_cast<float2*>(workspace);
  prm.lse2 = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + stats);
  prm.scores = scores;
  prm.score_stride = score_stride;
  prm.prompt_mass = prompt_mass;
  if (d->dtype == MASKKV_BF16) {
    return d->d == 128 ? launch_score_t<bf16_t, 128>(prm, d->B, stream, events) : launch_score_t<bf16_t, 64>(prm, d->B, stream, events);
  }
  return d->d == 128 ? launch_score_t<float, 128>(prm, d->B, stream, events) : launch_score_t<float, 64>(prm, d->B, stream, events);
}

}  // namespace maskkv
