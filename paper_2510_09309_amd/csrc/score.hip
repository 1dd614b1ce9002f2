// Mask-Voting scoring kernels (MaskKV Section 3.3, Stage 1):
//   A = softmax_row(Q_mask K_full^T * scale),  I_j = sum_i A_ij over the prompt columns.
//
// A column sum needs every row's final softmax normaliser, so the logits are formed twice:
//   pass 1  row statistics (reference exponent and sum of exponentials, base 2) per key segment,
//   merge   per-row log-sum-exp over the segments (+ the prompt's share of each row = prompt mass),
//   pass 2  logits again, p = exp2(s*c - lse), summed over the queries for every prompt key.
// Storing the n_m x N logits instead would cost far more HBM traffic than the second MFMA pass.
//
// Work decomposition: the key axis of every (b, h) is cut into 64-key tiles (prompt tiles, then response
// tiles; a tile never straddles the prompt/response boundary).  All tiles of the launch form one global
// index space that is divided evenly over a grid of about two workgroups per compute unit, so every
// workgroup streams the same number of tiles whatever the batch raggedness.  A workgroup walks its range
// as "segments" (maximal runs inside one region of one head).  More than 256 voting rows per head (long
// response spans, grouped-query heads) are cut into groups of 256; every (head, query group) pair has its own
// copy of the head's tiles in the index space, so a workgroup keeps one set of query fragments for a long run
// of tiles, and the groups' column sums are added in a fixed order by a last small kernel.
//
// Tiling: a workgroup holds the 256 voting rows of its query group as MFMA operands in registers - four waves
// of 64 queries, except bf16 pass 1, which runs eight waves of 32 (see ScoreCfg) - and K tiles stream through a
// padded, double-buffered LDS tile shared by its waves.  Pass 1 puts keys on the
// MFMA row axis so that a lane owns one query and the softmax statistics never leave the lane; pass 2
// puts queries on the row axis so that the sum over queries is in-lane adds plus one cross-lane exchange.
#include <type_traits>

#include "kernels.hpp"

namespace maskkv {

namespace {

constexpr int kQPerGroup = 256;                        // voting rows per query group
constexpr int kTargetGroups = 512;                     // about two resident workgroups per compute unit
constexpr double kSkew = 1.7;                          // tile share of an early workgroup relative to a late one
constexpr float kLazyLimit = 1.152921504606847e18f;    // 2^60: pass 1 re-centres its reference beyond this

template <typename T, int D, int PASS>
struct ScoreCfg {
  // Wave shape: bf16 pass 1 runs eight waves of 32 queries (four waves per SIMD with two workgroups per
  // compute unit; measured faster there), every other case four waves of 64 queries (two per SIMD).
  static constexpr int kNQ = (sizeof(T) == 2 && PASS == 1) ? 1 : 2;  // 32-query MFMA blocks per wave
  static constexpr int kWaves = kQPerGroup / (32 * kNQ);
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int kWavesPerSimd = kWaves / 2;
  static constexpr int kQPerWave = 32 * kNQ;
  static constexpr int kRowB = D * (int)sizeof(T);     // bytes per K row
  static constexpr int kRowP = kRowB + 16;             // padded LDS row: conflict-free 16-byte reads
  static constexpr int kSteps = kRowB / 32;            // fragments per row
  static constexpr int kTK = 64;                       // keys per tile: two 32-key blocks
  static constexpr int kPieces = kTK * kRowB / 16 / kThreads;  // 16-byte pieces per thread per tile
  static constexpr int kPiecesPerRow = kRowB / 16;
  static constexpr int kTileBytes = kTK * kRowP;
  static constexpr int kLdsBytes = 2 * kTileBytes;     // double-buffered K tile (dynamic LDS)
};

// Tile bookkeeping of one pass, computed on the host.
struct TileMap {
  int tk;                         // keys per tile
  int with_resp;                  // 1: response tiles are part of the index space (pass 1)
  int R;                          // tiles per workgroup, first G1 workgroups
  int R2;                         // tiles per workgroup, the others (R2 <= R)
  int G1;                         // see make_map
  int G;                          // workgroups in total
  __host__ __device__ int first_tile(int g) const { return g < G1 ? g * R : G1 * R + (g - G1) * R2; }
  __host__ __device__ int group_of(int tile) const { return tile < G1 * R ? tile / R : G1 + (tile - G1 * R) / R2; }
  int T;                          // tiles in total
  int nqg;                        // query groups per head: every (head, group) pair owns a copy of the head's tiles
  int toff[MASKKV_MAX_BATCH + 1]; // first global tile of sequence b (all its heads and query groups)
};

struct ScoreParams {
  View Q, K;
  Lens lens;
  TileMap map;        // of the pass being launched
  TileMap map1;       // of pass 1 (the merge kernel needs it to find the partial statistics)
  int B, H, n_resp;
  int n_query;        // voting rows per key/value head: q_per_kv query heads of n_qh mask queries each
  int n_qh, q_per_kv;
  int parts_p, parts_r;  // partial-statistics slots per (b, h): prompt region, response region
  float c;            // scale * log2(e)
  float2* stats;      // [B*H][parts_p + parts_r][n_query] (reference, sum) in the base-2 domain
  float* lse2;        // [B*H][n_query]
  const float* row_lse;  // [B*H][n_query] natural-log normalisers given by the caller (then pass 1 is not run), or null
  float* scores;      // [B*H][score_stride]
  int64_t score_stride;
  float* group_sums;  // [B*H][nqg][group_stride] column sums per query group (more than one group only)
  int64_t group_stride;
  float* prompt_mass; // [B*H] or null
};

__device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }

template <typename T, int D, int PASS>
__device__ __forceinline__ void load_tile_global(const char* kbase, int64_t stride_t, int key0, int klast,
                                                 u32x4 (&regs)[ScoreCfg<T, D, PASS>::kPieces]) {
  using C = ScoreCfg<T, D, PASS>;
#pragma unroll
  for (int i = 0; i < C::kPieces; ++i) {
    const int p = threadIdx.x + i * C::kThreads;
    const int row = p / C::kPiecesPerRow;
    const int col = p % C::kPiecesPerRow;
    const int key = min(key0 + row, klast);  // rows past the segment end re-read its last valid row
    regs[i] = *reinterpret_cast<const u32x4*>(kbase + (int64_t)key * stride_t + col * 16);
  }
}

template <typename T, int D, int PASS>
__device__ __forceinline__ void store_tile_lds(char* buf, const u32x4 (&regs)[ScoreCfg<T, D, PASS>::kPieces]) {
  using C = ScoreCfg<T, D, PASS>;
#pragma unroll
  for (int i = 0; i < C::kPieces; ++i) {
    const int p = threadIdx.x + i * C::kThreads;
    const int row = p / C::kPiecesPerRow;
    const int col = p % C::kPiecesPerRow;
    *reinterpret_cast<u32x4*>(buf + row * C::kRowP + col * 16) = regs[i];
  }
}

// PASS 1: row statistics.  PASS 2: column sums.
template <typename T, int D, int PASS>
__global__ __launch_bounds__((ScoreCfg<T, D, PASS>::kThreads), (ScoreCfg<T, D, PASS>::kWavesPerSimd)) void score_kernel(const ScoreParams prm) {
  using C = ScoreCfg<T, D, PASS>;
  extern __shared__ __attribute__((aligned(16))) char kt_raw[];  // two K tiles
  __shared__ float cs[3][C::kWaves][C::kTK];  // pass 2: per-wave column partials of the last three tiles
  __shared__ float nlse[kQPerGroup];            // pass 2: -lse2 of the current query group

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int r = lane & 31;
  const int g = lane >> 5;
  const float c = prm.c;
  const float inv_c = 1.0f / c;
  const TileMap& map = prm.map;

  int s = map.first_tile(blockIdx.x);
  const int e = min(map.T, map.first_tile(blockIdx.x + 1));
  int cur_bh = -1, cur_qg = -1;
  u32x4 qf[C::kNQ][C::kSteps];
  f32x16 nb[C::kNQ];  // pass 2: -lse2 / c of this lane's query rows, the initial value of every logits block

  while (s < e) {
    // ---- locate the segment that starts at global tile s
    int b = 0;
    while (b + 1 < prm.B && map.toff[b + 1] <= s) ++b;
    const int P = prm.lens.P[b];
    const int npt = ceil_div(P, C::kTK);
    const int nrt = ceil_div(prm.n_resp, C::kTK);
    const int tiles_h = map.with_resp ? npt + nrt : npt;
    const int rem = s - map.toff[b];
    const int hv = rem / tiles_h;  // (head, query group) pair
    const int h = hv / map.nqg;
    const int qgi = hv - h * map.nqg;
    const int qg = qgi * kQPerGroup;
    const int t_in = rem - hv * tiles_h;
    const bool prompt = t_in < npt;
    const int head0 = map.toff[b] + hv * tiles_h;
    const int region_start = head0 + (prompt ? 0 : npt);
    const int region_end = head0 + (prompt ? npt : tiles_h);
    const int seg_end = min(e, region_end);
    const int nt = seg_end - s;
    const int k0 = (prompt ? 0 : P) + (s - region_start) * C::kTK;
    const int k1 = min(prompt ? P : P + prm.n_resp, k0 + nt * C::kTK);
    const int bh = b * prm.H + h;
    const char* kbase = prm.K.row(b, h, 0);
    const int64_t kstride = prm.K.stride_t;

    {
      const int q0 = qg + wave * C::kQPerWave;
      const bool new_head = bh != cur_bh || qg != cur_qg;
      // Loads return in the order of their issue.  (Pass 2, on entering a head) this thread's row normaliser is asked
      // for first - the first barrier below waits for it and for nothing else - then the segment's first K tile,
      // then the query fragments, which are not needed before the first MFMA.
      float my_nlse = 0.f;
      if (PASS == 2 && new_head && (int)threadIdx.x < kQPerGroup) {
        const int q = qg + (int)threadIdx.x;
        my_nlse = q >= prm.n_query ? -INFINITY
                  : prm.row_lse    ? -prm.row_lse[(int64_t)bh * prm.n_query + q] * kLog2e
                                   : -prm.lse2[(int64_t)bh * prm.n_query + q];
      }
      u32x4 stage[C::kPieces];
      load_tile_global<T, D, PASS>(kbase, kstride, k0, k1 - 1, stage);
      if (new_head) {
        cur_bh = bh;
        cur_qg = qg;
        // Query fragments stay in registers for as long as the walk stays in this head.  Rows past
        // n_query re-read the last query: their statistics are never stored (pass 1) and their
        // probabilities are forced to zero through nb = -inf (pass 2).
#pragma unroll
        for (int blk = 0; blk < C::kNQ; ++blk) {
          const int q = min(q0 + blk * 32 + r, prm.n_query - 1);
          const char* qrow = prm.Q.group_row(b, h, prm.q_per_kv, prm.n_qh, q);
#pragma unroll
          for (int ks = 0; ks < C::kSteps; ++ks)
            qf[blk][ks] = *reinterpret_cast<const u32x4*>(qrow + ks * 32 + g * 16);
        }
        if (PASS == 2) {
          __syncthreads();
          if ((int)threadIdx.x < kQPerGroup) nlse[threadIdx.x] = my_nlse;
          __syncthreads();
          // (one reciprocal instead of 32 divisions, each a chain of about ten dependent instructions; the start
          // value moves by one ulp at most, a probability by 1e-6 relative)
#pragma unroll
          for (int blk = 0; blk < C::kNQ; ++blk)
#pragma unroll
            for (int i = 0; i < 16; ++i) nb[blk][i] = nlse[wave * C::kQPerWave + blk * 32 + 8 * (i / 4) + 4 * g + (i % 4)] * inv_c;
        }
      }

      // pass 1 state: this lane's (reference exponent, sum) for query q0 + 32*blk + r over the keys it sees
      float run_m[C::kNQ], run_l[C::kNQ];
#pragma unroll
      for (int blk = 0; blk < C::kNQ; ++blk) {
        run_m[blk] = kNegBig;
        run_l[blk] = 0.f;
      }

      float* out = map.nqg == 1 ? prm.scores + (int64_t)bh * prm.score_stride
                                : prm.group_sums + ((int64_t)bh * map.nqg + qgi) * prm.group_stride;
      auto flush = [&](int t) {  // tile t of this segment: add the waves' partials, write the column sums
        const int j = k0 + t * C::kTK + (int)threadIdx.x;
        if ((int)threadIdx.x < C::kTK && j < k1) {
          float v = 0.f;
#pragma unroll
          for (int w = 0; w < C::kWaves; ++w) v += cs[t % 3][w][threadIdx.x];
          out[j] = v;
        }
      };

      // Logits of one 32-key block (both 32-query blocks of this wave) on the matrix pipe.
      auto form = [&](const char* buf, int kb, f32x16 (&a)[C::kNQ]) {
        // Pass 2 starts every block from -lse/c of its query rows: the matrix pipe then delivers s - lse/c
        // and the vector pipe is left with one multiply, one exponential and one add per logit.
#pragma unroll
        for (int blk = 0; blk < C::kNQ; ++blk) a[blk] = PASS == 2 ? nb[blk] : f32x16{};
#pragma unroll
        for (int ks = 0; ks < C::kSteps; ++ks) {
          const u32x4 kf = *reinterpret_cast<const u32x4*>(buf + (kb * 32 + r) * C::kRowP + ks * 32 + g * 16);
#pragma unroll
          for (int blk = 0; blk < C::kNQ; ++blk) {
            if (PASS == 1)
              mfma_step<T>(kf, qf[blk][ks], a[blk]);  // S^T block: keys on rows, queries on columns
            else
              mfma_step<T>(qf[blk][ks], kf, a[blk]);  // S block: queries on rows, keys on columns
          }
        }
      };
      // Exponentials and sums of one formed block on the vector pipe.  MASKED is only needed for the last
      // tile of a segment (rows past the segment end re-read its last row and must not be counted).
      auto reduce = [&](auto masked, int t, int kb, f32x16 (&a)[C::kNQ]) {
        if (PASS == 1) {
          if (decltype(masked)::value) {
            const int nvalid = k1 - (k0 + t * C::kTK + kb * 32);  // rows >= nvalid are past the segment end
#pragma unroll
            for (int blk = 0; blk < C::kNQ; ++blk)
#pragma unroll
              for (int i = 0; i < 16; ++i)
                if (8 * (i / 4) + 4 * g + (i % 4) >= nvalid) a[blk][i] = -INFINITY;
          }
          // Exponentials against the current reference; the reference is only moved (slow path) when a sum
          // leaves the safe range, which also covers the very first block (reference = -1e30).  One
          // branch per stage, after all the vector work, keeps the fast path a single basic block.
          float sum[C::kNQ];
          bool ok = true;
#pragma unroll
          for (int blk = 0; blk < C::kNQ; ++blk) {
            sum[blk] = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) sum[blk] += fast_exp2(fmaf(a[blk][i], c, -run_m[blk]));
            ok = ok && sum[blk] < kLazyLimit;
          }
          if (__all(ok)) {
#pragma unroll
            for (int blk = 0; blk < C::kNQ; ++blk) run_l[blk] += sum[blk];
          } else {
#pragma unroll
            for (int blk = 0; blk < C::kNQ; ++blk) {
              float bm = a[blk][0];
#pragma unroll
              for (int i = 1; i < 16; ++i) bm = fmaxf(bm, a[blk][i]);
              const float m_new = fmaxf(run_m[blk], bm * c);
              float s2 = 0.f;
#pragma unroll
              for (int i = 0; i < 16; ++i) s2 += fast_exp2(fmaf(a[blk][i], c, -m_new));
              run_l[blk] = run_l[blk] * fast_exp2(run_m[blk] - m_new) + s2;
              run_m[blk] = m_new;
            }
          }
        } else {
          float colsum = 0.f;
#pragma unroll
          for (int blk = 0; blk < C::kNQ; ++blk)
#pragma unroll
            for (int i = 0; i < 16; ++i) colsum += fast_exp2(a[blk][i] * c);
          colsum += xor32(colsum);
          if (g == 0) cs[t % 3][wave][kb * 32 + r] = colsum;
        }
      };

      // Software pipeline inside every wave: while the matrix pipe forms block n+1 into one accumulator
      // pair, the vector pipe reduces block n from the other pair (both in one basic block, so that the
      // compiler interleaves MFMA and VALU issue).  A tile holds blocks (t,0) and (t,1):
      //   stage 1 of iteration t: form (t,1) -> B  |  reduce (t,0) from A
      //   tile t+1: registers -> LDS, barrier, request tile t+2 from global memory
      //   stage 2 of iteration t: form (t+1,0) -> A  |  reduce (t,1) from B
      f32x16 accA[C::kNQ], accB[C::kNQ];
      __syncthreads();  // the previous segment's readers are done with the tile and partial buffers
      store_tile_lds<T, D, PASS>(kt_raw, stage);
      if (nt > 1) load_tile_global<T, D, PASS>(kbase, kstride, k0 + C::kTK, k1 - 1, stage);
      __syncthreads();
      form(kt_raw, 0, accA);

      auto iteration = [&](auto masked, int t) {
        form(kt_raw + (t & 1) * C::kTileBytes, 1, accB);
        reduce(masked, t, 0, accA);
        if (t + 1 < nt) store_tile_lds<T, D, PASS>(kt_raw + ((t + 1) & 1) * C::kTileBytes, stage);
        __syncthreads();  // tile t+1 is visible; every wave is done reading tile t-1 and reducing into cs[(t-1)%3]
        if (t + 2 < nt) load_tile_global<T, D, PASS>(kbase, kstride, k0 + (t + 2) * C::kTK, k1 - 1, stage);
        if (PASS == 2 && t > 0) flush(t - 1);
        if (t + 1 < nt) form(kt_raw + ((t + 1) & 1) * C::kTileBytes, 0, accA);
        reduce(masked, t, 1, accB);
      };
      for (int t = 0; t + 1 < nt; ++t) iteration(std::false_type{}, t);
      if (PASS == 1 && k1 - k0 < nt * C::kTK)
        iteration(std::true_type{}, nt - 1);  // partial last tile
      else
        iteration(std::false_type{}, nt - 1);
      if (PASS == 2) {
        __syncthreads();
        flush(nt - 1);
      }

      if (PASS == 1) {
        const int part = (int)blockIdx.x - map.group_of(region_start);
        const int slot = bh * (prm.parts_p + prm.parts_r) + (prompt ? 0 : prm.parts_p) + part;
#pragma unroll
        for (int blk = 0; blk < C::kNQ; ++blk) {
          const float m_o = xor32(run_m[blk]);
          const float l_o = xor32(run_l[blk]);
          const float m = fmaxf(run_m[blk], m_o);
          const float l = run_l[blk] * fast_exp2(run_m[blk] - m) + l_o * fast_exp2(m_o - m);
          const int q = q0 + blk * 32 + r;
          if (g == 0 && q < prm.n_query) prm.stats[(int64_t)slot * prm.n_query + q] = make_float2(m, l);
        }
      }
    }
    s = seg_end;
  }
}

// Merge the per-segment statistics of every query row into its base-2 log-sum-exp; the prompt segments'
// share of each row's normaliser, summed over the rows, is the mask-to-prompt attention mass.
__global__ __launch_bounds__(256) void score_merge_kernel(const ScoreParams prm) {
  __shared__ float red[256];
  const TileMap& map = prm.map1;
  const int bh = blockIdx.x;
  const int b = bh / prm.H;
  const int h = bh % prm.H;
  const int P = prm.lens.P[b];
  const int npt = ceil_div(P, map.tk);
  const int nrt = ceil_div(prm.n_resp, map.tk);
  const int nslot = prm.parts_p + prm.parts_r;
  float mass = 0.f;
  for (int q = threadIdx.x; q < prm.n_query; q += 256) {
    // the tiles of this row's (head, query group) pair, and the workgroups of pass 1 that touched them
    const int a_p = map.toff[b] + (h * map.nqg + q / kQPerGroup) * (npt + nrt);
    const int a_r = a_p + npt;
    const int np_parts = npt > 0 ? map.group_of(a_p + npt - 1) - map.group_of(a_p) + 1 : 0;
    const int nr_parts = map.group_of(a_r + nrt - 1) - map.group_of(a_r) + 1;
    const float2* st = prm.stats + (int64_t)bh * nslot * prm.n_query + q;
    // One sweep over the slots, eight independent loads at a time; (M, Lp, Lr) are rescaled on the fly.
    float M = kNegBig, Lp = 0.f, Lr = 0.f;
    auto sweep = [&](int first, int count, float& L) {
      for (int i0 = 0; i0 < count; i0 += 8) {
        float2 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          v[u] = i0 + u < count ? st[(int64_t)(first + i0 + u) * prm.n_query] : make_float2(kNegBig, 0.f);
        float m8 = v[0].x;
#pragma unroll
        for (int u = 1; u < 8; ++u) m8 = fmaxf(m8, v[u].x);
        if (m8 > M) {
          const float f = fast_exp2(M - m8);
          Lp *= f;
          Lr *= f;
          M = m8;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) L += v[u].y * fast_exp2(v[u].x - M);
      }
    };
    sweep(0, np_parts, Lp);
    sweep(prm.parts_p, nr_parts, Lr);
    const float L = Lp + Lr;
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

// More than one query group: scores = sum of the groups' column sums, added in group order.
__global__ __launch_bounds__(256) void score_group_sum_kernel(const ScoreParams prm, int nqg) {
  const int bh = blockIdx.y;
  const int P = prm.lens.P[bh / prm.H];
  const int j = (int)blockIdx.x * 256 + (int)threadIdx.x;
  if (j >= P) return;
  const float* src = prm.group_sums + (int64_t)bh * nqg * prm.group_stride + j;
  float v = src[0];
  for (int i = 1; i < nqg; ++i) v += src[(int64_t)i * prm.group_stride];
  prm.scores[(int64_t)bh * prm.score_stride + j] = v;
}

// Prompt mass as the sum of a head's scores (the column sums of the prompt columns add up to the prompt's share of
// the voting rows' attention), for calls that do not run pass 1: one 1024-thread workgroup per (b, h), eight
// independent loads in flight per thread, fixed summation order.
constexpr int kMassThreads = 1024;

__global__ __launch_bounds__(kMassThreads) void score_mass_kernel(const ScoreParams prm) {
  __shared__ float red[kMassThreads];
  const int bh = blockIdx.x;
  const int P = prm.lens.P[bh / prm.H];
  const float* row = prm.scores + (int64_t)bh * prm.score_stride;
  float acc = 0.f;
  for (int j0 = threadIdx.x; j0 < P; j0 += 8 * kMassThreads) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int j = j0 + u * kMassThreads;
      v[u] = j < P ? row[j] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = kMassThreads / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) prm.prompt_mass[bh] = red[0];
}

int tile_keys(const maskkv_desc*) { return 64; }  // every configuration uses 64-key tiles

int query_groups(const maskkv_desc* d) {
  return (int)(((int64_t)d->n_query * query_heads_per_kv(d) + kQPerGroup - 1) / kQPerGroup);
}

int64_t group_stride(const maskkv_desc* d) { return ((int64_t)d->P_max + 63) / 64 * 64; }

TileMap make_map(const maskkv_desc* d, const Lens& lens, bool with_resp) {
  TileMap m;
  m.tk = tile_keys(d);
  m.with_resp = with_resp ? 1 : 0;
  m.nqg = query_groups(d);
  int t = 0;
  for (int b = 0; b <= MASKKV_MAX_BATCH; ++b) m.toff[b] = 0;
  for (int b = 0; b < d->B; ++b) {
    m.toff[b] = t;
    const int per_head = (lens.P[b] + m.tk - 1) / m.tk + (with_resp ? (d->n_resp + m.tk - 1) / m.tk : 0);
    t += per_head * d->H * m.nqg;
  }
  for (int b = d->B; b <= MASKKV_MAX_BATCH; ++b) m.toff[b] = t;
  m.T = t;
  // About two workgroups per compute unit are launched and all are resident at once.  The hardware favours
  // the older of the two workgroups that share a compute unit, so with equal shares the first half of the
  // grid finishes early and the second half then runs alone at lower efficiency: the first G1 workgroups
  // (one per compute unit in dispatch order) get kSkew times the tiles of the others (1.7 measured best at the
  // 32k-prompt shape: both halves then finish within a few percent of each other).
  m.G1 = kTargetGroups / 2;
  m.R2 = (int)((double)t / (m.G1 * (1.0 + kSkew)) + 0.999);
  if (m.R2 < 1) m.R2 = 1;
  m.R = (t - m.G1 * m.R2 + m.G1 - 1) / m.G1;
  if (m.R < m.R2) m.R = m.R2;
  m.G = t <= m.G1 * m.R ? (t + m.R - 1) / m.R : m.G1 + (t - m.G1 * m.R + m.R2 - 1) / m.R2;
  return m;
}

// Partial-statistics slots per (b, h): a region of n tiles is touched by at most ceil(n/R)+1 workgroups.
void stat_slots(const maskkv_desc* d, const Lens& lens, const TileMap& map1, int* parts_p, int* parts_r) {
  int npt_max = 0;
  for (int b = 0; b < d->B; ++b) npt_max = max(npt_max, (lens.P[b] + map1.tk - 1) / map1.tk);
  const int nrt = (d->n_resp + map1.tk - 1) / map1.tk;
  *parts_p = (npt_max + map1.R2 - 1) / map1.R2 + 1;
  *parts_r = (nrt + map1.R2 - 1) / map1.R2 + 1;
}

int mark(void* const* events, int i, hipStream_t stream) {
  if (!events || !events[i]) return MASKKV_OK;
  const hipError_t e = hipEventRecord(reinterpret_cast<hipEvent_t>(events[i]), stream);
  if (e == hipSuccess) return MASKKV_OK;
  set_error("score: hipEventRecord(events[%d]): %s", i, hipGetErrorString(e));
  return MASKKV_EHIP;
}

template <typename T, int D, int PASS>
int launch_pass(const ScoreParams& prm, hipStream_t stream) {
  using C = ScoreCfg<T, D, PASS>;
  static bool raised = false;  // one-time opt-in to more than the default dynamic LDS size
  if (C::kLdsBytes > 48 * 1024 && !raised) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_kernel<T, D, PASS>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
    if (e != hipSuccess) {
      set_error("score: cannot raise dynamic LDS limit: %s", hipGetErrorString(e));
      (void)hipGetLastError();
      return MASKKV_EHIP;
    }
    raised = true;
  }
  const dim3 grid(prm.map.G);
  hipLaunchKernelGGL((score_kernel<T, D, PASS>), grid, dim3(C::kThreads), C::kLdsBytes, stream, prm);
  return check_launch(PASS == 1 ? "score pass 1" : "score pass 2");
}

template <typename T, int D>
int launch_score_t(ScoreParams& prm, const TileMap& map2, hipStream_t stream, void* const* events) {
  if (int e = mark(events, 0, stream)) return e;
  if (!prm.row_lse) {
    prm.map = prm.map1;
    if (int e = launch_pass<T, D, 1>(prm, stream)) return e;
    if (int e = mark(events, 1, stream)) return e;
    hipLaunchKernelGGL(score_merge_kernel, dim3(prm.B * prm.H), dim3(256), 0, stream, prm);
    if (int e = check_launch("score merge")) return e;
    if (int e = mark(events, 2, stream)) return e;
  }
  if (map2.T > 0) {
    prm.map = map2;
    if (int e = launch_pass<T, D, 2>(prm, stream)) return e;
    if (map2.nqg > 1) {
      const dim3 grid((unsigned)((prm.group_stride + 255) / 256), prm.B * prm.H);
      hipLaunchKernelGGL(score_group_sum_kernel, grid, dim3(256), 0, stream, prm, map2.nqg);
      if (int e = check_launch("score (group sums)")) return e;
    }
  }
  if (prm.row_lse && prm.prompt_mass) {
    hipLaunchKernelGGL(score_mass_kernel, dim3(prm.B * prm.H), dim3(kMassThreads), 0, stream, prm);
    if (int e = check_launch("score (prompt mass)")) return e;
  }
  return mark(events, 3, stream);
}

}  // namespace

size_t score_workspace_bytes(const maskkv_desc* d, const Lens& lens) {
  int pp, pr;
  stat_slots(d, lens, make_map(d, lens, true), &pp, &pr);
  const int64_t bh = (int64_t)d->B * d->H;
  const int64_t nq = (int64_t)d->n_query * query_heads_per_kv(d);
  size_t stats = (size_t)(bh * (pp + pr) * nq) * sizeof(float2);
  stats = (stats + 255) / 256 * 256;
  const size_t lse = ((size_t)(bh * nq) * sizeof(float) + 255) / 256 * 256;
  const int nqg = query_groups(d);
  const size_t sums = nqg > 1 ? (size_t)(bh * nqg * group_stride(d)) * sizeof(float) : 0;
  return stats + lse + sums;
}

int launch_score(const maskkv_desc* d, const View& Q, const View& K, const Lens& lens, float scale, float* scores,
                 int64_t score_stride, float* prompt_mass, void* workspace, hipStream_t stream,
                 void* const* events, const float* row_lse) {
  ScoreParams prm;
  prm.row_lse = row_lse;
  prm.Q = Q;
  prm.K = K;
  prm.lens = lens;
  prm.map1 = make_map(d, lens, true);
  const TileMap map2 = make_map(d, lens, false);
  prm.B = d->B;
  prm.H = d->H;
  prm.n_resp = d->n_resp;
  prm.q_per_kv = query_heads_per_kv(d);
  prm.n_qh = d->n_query;
  prm.n_query = d->n_query * prm.q_per_kv;
  stat_slots(d, lens, prm.map1, &prm.parts_p, &prm.parts_r);
  prm.c = scale * kLog2e;
  const int64_t bh = (int64_t)d->B * d->H;
  size_t stats = (size_t)(bh * (prm.parts_p + prm.parts_r) * prm.n_query) * sizeof(float2);
  stats = (stats + 255) / 256 * 256;
  prm.stats = reinterpret_cast<float2*>(workspace);
  prm.lse2 = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + stats);
  const size_t lse = ((size_t)(bh * prm.n_query) * sizeof(float) + 255) / 256 * 256;
  prm.group_sums = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + stats + lse);
  prm.group_stride = group_stride(d);
  prm.scores = scores;
  prm.score_stride = score_stride;
  prm.prompt_mass = prompt_mass;
  if (d->dtype == MASKKV_BF16)
    return d->d == 128 ? launch_score_t<bf16_t, 128>(prm, map2, stream, events)
                       : launch_score_t<bf16_t, 64>(prm, map2, stream, events);
  return d->d == 128 ? launch_score_t<float, 128>(prm, map2, stream, events)
                     : launch_score_t<float, 64>(prm, map2, stream, events);
}

}  // namespace maskkv
