// Bidirectional attention of the response span over [kept prompt KV ; response KV]
// (MaskKV Section 3.1 layer forward equation; appendix: AttnOut_m = sum_j alpha_mj V_j), and the
// same attention over the un-evicted sequence.
//
// Flash-style single pass with an online softmax.  One workgroup = 8 waves = 256 queries of one (b, h)
// sharing every staged K/V tile (4 waves at bf16 head_dim 64); each wave owns 32 queries.  The logits are formed transposed (keys on the MFMA row axis, queries on
// the column axis), so a lane owns one query: its running max / sum stay in the lane and the
// probabilities it holds are already laid out as the B operand of O^T = V^T P^T.  V tiles are written
// to LDS transposed so that the A operand of that product is read with 8/16-byte LDS loads.
// The key axis is the concatenation of two segments (packed cache rows, then a strided view); long key
// axes are split across workgroups and merged by a second small kernel.
#include "kernels.hpp"

namespace maskkv {

namespace {

// Launches of fewer 128-query tiles than this take the narrow kernel (measured at 256 queries and about 512 keys
// per head: 32 heads 17 vs 30 us, 64 heads 30 vs 31 us, 96 heads 44 vs 32 us for narrow vs tiled).
constexpr int kNarrowBelow = 144;
constexpr float kLazyBump = 8.f;  // log2 of the largest probability tolerated before the running reference is raised

template <typename T, int D>
struct AttCfg {
  static constexpr int kRowB = D * (int)sizeof(T);
  static constexpr int kRowP = kRowB + 16;
  static constexpr int kSteps = kRowB / 32;
  static constexpr int kTK = (kRowB <= 256) ? 64 : 32;
  static constexpr int kNKB = kTK / 32;
  static constexpr int kPiecesPerRow = kRowB / 16;
  // Waves (32 queries each) that share a K/V tile: eight where a thread still moves whole 16-byte pieces of K
  // and pairs of V rows, i.e. everywhere but bf16 at head_dim 64.
  static constexpr int kWaves = (sizeof(T) == 2 && D == 64) ? 4 : 8;
  static constexpr int kThreads = kWaves * 64;
  static constexpr int kQPerBlock = kWaves * 32;
  static constexpr int kPieces = kTK * kRowB / 16 / kThreads;
  static constexpr int kSV = kTK + 4;  // elements per transposed-V row (padding keeps LDS reads conflict-free)
  // bf16: every group of 32 transposed-V rows is shifted by a further 16 bytes.  The fragment reads of a wave stay
  // inside one group and are unaffected; the transposing stores of a wave touch one row of every group, which
  // without the shift fall on the same LDS banks four at a time.
  static constexpr int kVGroupShift = sizeof(T) == 2 ? 16 : 0;
  static constexpr int kDB = D / 32;
  static constexpr int kKtBytes = kTK * kRowP;
  static constexpr int kVtBytes = D * kSV * (int)sizeof(T) + (D / 32) * kVGroupShift;
  static constexpr int kLds = 2 * (kKtBytes + kVtBytes);  // K and V^T tiles, double-buffered
};

struct AttendParams {
  View Q, K2, V2, O;
  Lens lens;
  const char* Kc;
  const char* Vc;
  const int32_t* cu;
  int64_t capacity;
  int H, BH, n_resp, full, n_splits;
  int q_per_kv;  // query heads per key/value head
  int n_q;       // query rows per key/value head = q_per_kv * n_resp
  float c;  // scale * log2(e)
  float* lse;
  const int32_t* order;  // [BH] heads by descending key count (compressed call of the tiled kernel), or null
  float* part_o;     // [BH][n_splits][n_q][D]
  float2* part_ml;   // [BH][n_splits][n_q]
};

struct KeySpace {
  const char* a_k;  // packed segment base (row 0 of this head), rows contiguous
  const char* a_v;
  int len_a;
  int len_b;
};

template <typename T, int D>
__device__ __forceinline__ void load_kv(const AttendParams& prm, const KeySpace& ks, int b, int h, int key0, int klast,
                                        u32x4 (&kr)[AttCfg<T, D>::kPieces], u32x4 (&vr)[AttCfg<T, D>::kPieces]) {
  using C = AttCfg<T, D>;
#pragma unroll
  for (int i = 0; i < C::kPieces; ++i) {
    const int p = threadIdx.x + i * C::kThreads;
    {
      const int row = p / C::kPiecesPerRow, col = p % C::kPiecesPerRow;
      const int j = min(key0 + row, klast);
      const char* src = j < ks.len_a ? ks.a_k + (int64_t)j * C::kRowB : prm.K2.row(b, h, j - ks.len_a);
      kr[i] = *reinterpret_cast<const u32x4*>(src + col * 16);
    }
    {
      int row, col;
      if (sizeof(T) == 2) {  // item = (key pair, 16-byte slice); pieces 2i and 2i+1 are the pair's two rows
        const int item = threadIdx.x + (i / 2) * C::kThreads;
        row = 2 * (item / C::kPiecesPerRow) + (i & 1);
        col = item % C::kPiecesPerRow;
      } else {
        row = p / C::kPiecesPerRow;
        col = p % C::kPiecesPerRow;
      }
      const int j = min(key0 + row, klast);
      const char* src = j < ks.len_a ? ks.a_v + (int64_t)j * C::kRowB : prm.V2.row(b, h, j - ks.len_a);
      vr[i] = *reinterpret_cast<const u32x4*>(src + col * 16);
    }
  }
}

template <typename T, int D>
__device__ __forceinline__ void store_kv(char* kt, char* vt, const u32x4 (&kr)[AttCfg<T, D>::kPieces],
                                         const u32x4 (&vr)[AttCfg<T, D>::kPieces]) {
  using C = AttCfg<T, D>;
#pragma unroll
  for (int i = 0; i < C::kPieces; ++i) {
    const int p = threadIdx.x + i * C::kThreads;
    const int row = p / C::kPiecesPerRow, col = p % C::kPiecesPerRow;
    *reinterpret_cast<u32x4*>(kt + row * C::kRowP + col * 16) = kr[i];
  }
  uint32_t* vt32 = reinterpret_cast<uint32_t*>(vt);
  if (sizeof(T) == 2) {
    // vt[e][key] as bf16: a 32-bit word holds keys (2*pair, 2*pair+1) of one head-dim element
#pragma unroll
    for (int i = 0; i < C::kPieces / 2; ++i) {
      const int item = threadIdx.x + i * C::kThreads;
      const int pair = item / C::kPiecesPerRow, col = item % C::kPiecesPerRow;
      const u32x4 a = vr[2 * i], bq = vr[2 * i + 1];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t lo = (a[w] & 0xFFFFu) | (bq[w] << 16);
        const uint32_t hi = (a[w] >> 16) | (bq[w] & 0xFFFF0000u);
        const int row = col * 8 + 2 * w;
        const int word = row * (C::kSV / 2) + (row / 32) * (C::kVGroupShift / 4) + pair;  // (row is even)
        vt32[word] = lo;
        vt32[word + C::kSV / 2] = hi;
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < C::kPieces; ++i) {
      const int p = threadIdx.x + i * C::kThreads;
      const int row = p / C::kPiecesPerRow, col = p % C::kPiecesPerRow;
#pragma unroll
      for (int w = 0; w < 4; ++w) vt32[(col * 4 + w) * C::kSV + row] = vr[i][w];
    }
  }
}

template <typename T, int D>
__global__ __launch_bounds__((AttCfg<T, D>::kThreads)) void attend_kernel(const AttendParams prm) {
  using C = AttCfg<T, D>;
  extern __shared__ __attribute__((aligned(16))) char att_lds[];  // two buffers of (K tile, V^T tile)

  // Workgroup numbers that are congruent modulo 8 run on the same XCD and share its L2.  The query tiles of
  // one (head, key split) read the same K/V rows, so they are given consecutive slots of one XCD: the rows
  // then come from HBM once instead of once per query tile.
  const int qtiles = (prm.n_q + C::kQPerBlock - 1) / C::kQPerBlock;
  const int slot = blockIdx.x / 8;
  const int unit = (slot / qtiles) * 8 + blockIdx.x % 8;  // (head, split) pair
  const int qtile = slot % qtiles;
  if (unit >= prm.BH * prm.n_splits) return;
  const int bh = prm.order ? prm.order[unit] : unit / prm.n_splits;  // (an order is only given without splits)
  const int split = prm.order ? 0 : unit % prm.n_splits;
  const int b = bh / prm.H;
  const int h = bh % prm.H;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int r = lane & 31;
  const int g = lane >> 5;

  KeySpace ks;
  if (prm.full) {
    ks.a_k = ks.a_v = nullptr;
    ks.len_a = 0;
    ks.len_b = prm.lens.P[b] + prm.n_resp;
  } else {
    const int64_t c0 = min((int64_t)prm.cu[bh], prm.capacity);
    const int64_t c1 = min((int64_t)prm.cu[bh + 1], prm.capacity);
    ks.a_k = prm.Kc + c0 * C::kRowB;
    ks.a_v = prm.Vc + c0 * C::kRowB;
    ks.len_a = (int)(c1 - c0);
    ks.len_b = prm.n_resp;
  }
  const int Lk = ks.len_a + ks.len_b;
  const int Ls = ((Lk + prm.n_splits - 1) / prm.n_splits + C::kTK - 1) / C::kTK * C::kTK;
  const int j0 = split * Ls;
  const int j1 = min(Lk, j0 + Ls);
  const int ntiles = j1 > j0 ? (j1 - j0 + C::kTK - 1) / C::kTK : 0;

  const int q = qtile * C::kQPerBlock + wave * 32 + r;
  u32x4 qf[C::kSteps];
#pragma unroll
  for (int s = 0; s < C::kSteps; ++s) {
    if (q < prm.n_q)
      qf[s] = *reinterpret_cast<const u32x4*>(prm.Q.group_row(b, h, prm.q_per_kv, prm.n_resp, q) + s * 32 + g * 16);
    else
      qf[s] = u32x4{0u, 0u, 0u, 0u};
  }

  f32x16 o[C::kDB];
#pragma unroll
  for (int db = 0; db < C::kDB; ++db) o[db] = f32x16{};
  float m = kNegBig, l = 0.f;
  const float c = prm.c;

  // Two tiles are kept in flight in two register sets (a key axis of a few hundred rows is a short serial
  // chain of tiles, so the memory latency of each request has to hide behind two tiles of arithmetic).
  u32x4 kra[C::kPieces], vra[C::kPieces], krb[C::kPieces], vrb[C::kPieces];
  // Tile t is computed from LDS buffer t&1 while tile t+1 is written to the other one: one barrier per tile.
  if (ntiles > 0) load_kv<T, D>(prm, ks, b, h, j0, j1 - 1, kra, vra);
  if (ntiles > 1) load_kv<T, D>(prm, ks, b, h, j0 + C::kTK, j1 - 1, krb, vrb);
  if (ntiles > 0) {
    store_kv<T, D>(att_lds, att_lds + C::kKtBytes, kra, vra);
    if (ntiles > 2) load_kv<T, D>(prm, ks, b, h, j0 + 2 * C::kTK, j1 - 1, kra, vra);
  }
  __syncthreads();

  // `kr`, `vr` hold tile t+1 on entry (if there is one) and are refilled with tile t+3.
  auto tile_step = [&](int t, u32x4 (&kr)[C::kPieces], u32x4 (&vr)[C::kPieces]) {
    const int key0 = j0 + t * C::kTK;
    const char* kt = att_lds + (t & 1) * (C::kKtBytes + C::kVtBytes);
    const char* vt = kt + C::kKtBytes;
    if (t + 1 < ntiles) {  // the other buffer's readers (tile t-1) passed the barrier that ended the previous step
      char* nk = att_lds + ((t + 1) & 1) * (C::kKtBytes + C::kVtBytes);
      store_kv<T, D>(nk, nk + C::kKtBytes, kr, vr);
      if (t + 3 < ntiles) load_kv<T, D>(prm, ks, b, h, key0 + 3 * C::kTK, j1 - 1, kr, vr);
    }

    // S^T = K Q^T for this tile
    f32x16 s[C::kNKB];
#pragma unroll
    for (int kb = 0; kb < C::kNKB; ++kb) {
      s[kb] = f32x16{};
#pragma unroll
      for (int st = 0; st < C::kSteps; ++st) {
        const u32x4 kf = *reinterpret_cast<const u32x4*>(kt + (kb * 32 + r) * C::kRowP + st * 32 + g * 16);
        mfma_step<T>(kf, qf[st], s[kb]);
      }
      const int nvalid = j1 - (key0 + kb * 32);
      if (nvalid < 32) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (8 * (i / 4) + 4 * g + (i % 4) >= nvalid) s[kb][i] = -INFINITY;
      }
    }
    // online softmax; lanes l and l^32 hold the same query
    float bm = s[0][0];
#pragma unroll
    for (int kb = 0; kb < C::kNKB; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) bm = fmaxf(bm, s[kb][i]);
    bm = fmaxf(bm, xor32(bm));
    // The reference m is only raised when a tile exceeds it by more than 2^kLazyBump: probabilities then stay
    // below 2^kLazyBump (harmless in fp32 sums and as bf16 operands, whose exponent range is fp32's), and the
    // accumulators are rescaled on few tiles only.
    const float cand = bm * c;
    const bool bump = cand > m + kLazyBump;
    if (__any(bump)) {
      const float m_new = bump ? cand : m;
      const float alpha = fast_exp2(m - m_new);
      m = m_new;
      l *= alpha;
#pragma unroll
      for (int db = 0; db < C::kDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
    }
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < C::kNKB; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = fast_exp2(fmaf(s[kb][i], c, -m));
        s[kb][i] = p;
        psum += p;
      }
    l += psum;

    // O^T += V^T P^T
    if (sizeof(T) == 2) {
#pragma unroll
      for (int kb = 0; kb < C::kNKB; ++kb)
#pragma unroll
        for (int tp = 0; tp < 2; ++tp) {
          u32x4 pf;
#pragma unroll
          for (int w = 0; w < 4; ++w)
            pf[w] = pack_bf16x2(s[kb][8 * tp + 2 * w], s[kb][8 * tp + 2 * w + 1]);
#pragma unroll
          for (int db = 0; db < C::kDB; ++db) {
            const char* rowp = vt + ((db * 32 + r) * C::kSV + kb * 32 + 16 * tp + 4 * g) * 2 + db * C::kVGroupShift;
            const u32x2 lo = *reinterpret_cast<const u32x2*>(rowp);
            const u32x2 hi = *reinterpret_cast<const u32x2*>(rowp + 16);
            const u32x4 vf = {lo[0], lo[1], hi[0], hi[1]};
            mfma_step<T>(vf, pf, o[db]);
          }
        }
    } else {
#pragma unroll
      for (int kb = 0; kb < C::kNKB; ++kb)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          u32x4 pf;
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const float pv = s[kb][4 * qd + w];
            pf[w] = as_u32(pv);
          }
#pragma unroll
          for (int db = 0; db < C::kDB; ++db) {
            const u32x4 vf =
                *reinterpret_cast<const u32x4*>(vt + ((db * 32 + r) * C::kSV + kb * 32 + 8 * qd + 4 * g) * 4);
            mfma_step<T>(vf, pf, o[db]);
          }
        }
    }
    __syncthreads();  // tile t+1 is visible; every wave is done with tile t
  };
  for (int t = 0; t < ntiles; t += 2) {
    tile_step(t, krb, vrb);
    if (t + 1 < ntiles) tile_step(t + 1, kra, vra);
  }

  const float l_tot = l + xor32(l);
  if (q >= prm.n_q) return;
  if (prm.n_splits == 1) {
    const float inv = 1.f / l_tot;
    char* orow = prm.O.group_row(b, h, prm.q_per_kv, prm.n_resp, q);
#pragma unroll
    for (int db = 0; db < C::kDB; ++db)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        const int e = db * 32 + 8 * qd + 4 * g;
        const float v0 = o[db][4 * qd] * inv, v1 = o[db][4 * qd + 1] * inv;
        const float v2 = o[db][4 * qd + 2] * inv, v3 = o[db][4 * qd + 3] * inv;
        if (sizeof(T) == 2) {
          u32x2 w;
          w[0] = pack_bf16x2(v0, v1);
          w[1] = pack_bf16x2(v2, v3);
          *reinterpret_cast<u32x2*>(orow + e * 2) = w;
        } else {
          *reinterpret_cast<float4*>(orow + e * 4) = make_float4(v0, v1, v2, v3);
        }
      }
    if (prm.lse && g == 0) prm.lse[(int64_t)bh * prm.n_q + q] = (m + __log2f(l_tot)) * kLn2;
  } else {
    const int64_t slot = ((int64_t)bh * prm.n_splits + split) * prm.n_q + q;
    float* po = prm.part_o + slot * D;
#pragma unroll
    for (int db = 0; db < C::kDB; ++db)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        const int e = db * 32 + 8 * qd + 4 * g;
        *reinterpret_cast<float4*>(po + e) =
            make_float4(o[db][4 * qd], o[db][4 * qd + 1], o[db][4 * qd + 2], o[db][4 * qd + 3]);
      }
    if (g == 0) prm.part_ml[slot] = make_float2(m, l_tot);
  }
}

// ---------------------------------------------------------------------------------------------
// Narrow launches (few heads x query tiles, bf16): the kernel above would occupy a fraction of the compute
// units with one long serial chain of tiles each.  Here a workgroup serves 32 queries and its four waves
// split the key axis: wave w takes the 32-key blocks w, w+4, ... on its own - K fragments straight from
// global memory into registers, V through a wave-private transposed LDS tile, no workgroup barrier in the
// loop - and the four partial (O, m, l) are merged through LDS at the end.  Two blocks per wave are kept in
// flight.  Workgroups of one head are given indices that are congruent modulo 8, which places them on one
// XCD, so the head's K/V rows are fetched into one L2 only.
constexpr int kNarrowVS = 36;      // bf16 elements per transposed-V row: 32 keys + padding
constexpr int kNarrowShift = 16;   // bytes by which every group of 32 rows is shifted further (as in the tiled kernel)

// NW waves per workgroup split the key axis.
template <int D, int NW>
struct NarrowCfg {
  static constexpr int kThreads = 64 * NW;
  static constexpr int kRowB = D * 2;
  static constexpr int kSteps = kRowB / 32;
  static constexpr int kPPR = kRowB / 16;        // 16-byte pieces per row
  static constexpr int kVP = 32 * kPPR / 64;     // V pieces per lane per block
  static constexpr int kDB = D / 32;
  static constexpr int kVtBytes = D * kNarrowVS * 2 + (D / 32) * kNarrowShift;  // per wave
  static constexpr int kMergeBytes = NW * kDB * 16 * 64 * 4;        // partial O of the waves
  static constexpr int kLds = (kMergeBytes > NW * kVtBytes ? kMergeBytes : NW * kVtBytes) + NW * 32 * 8;
};

template <int D, int NW>
__global__ __launch_bounds__((NarrowCfg<D, NW>::kThreads)) void attend_narrow_kernel(const AttendParams prm) {
  using T = bf16_t;
  using C = NarrowCfg<D, NW>;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int nqt = (prm.n_q + 31) / 32;
  const int id = blockIdx.x;
  const int bh = (id / (8 * nqt)) * 8 + id % 8;
  const int qt = (id / 8) % nqt;
  if (bh >= prm.BH) return;
  const int b = bh / prm.H;
  const int h = bh % prm.H;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int r = lane & 31;
  const int g = lane >> 5;

  const int64_t c0 = min((int64_t)prm.cu[bh], prm.capacity);
  const int64_t c1 = min((int64_t)prm.cu[bh + 1], prm.capacity);
  const char* a_k = prm.Kc + c0 * C::kRowB;
  const char* a_v = prm.Vc + c0 * C::kRowB;
  const int len_a = (int)(c1 - c0);
  const int Lk = len_a + prm.n_resp;
  const int nblk = (Lk + 31) / 32;

  auto key_row = [&](const char* packed, const View& rest, int j) -> const char* {
    return j < len_a ? packed + (int64_t)j * C::kRowB : rest.row(b, h, j - len_a);
  };
  // Ask for block blk: K in MFMA fragment layout (lane = key row), V as row pieces for the transposition
  // (item = (key pair, 16-byte slice); pieces 2i and 2i+1 are the pair's two rows).  Rows past the end of
  // the key axis re-read its last row and are masked.
  auto request = [&](int blk, u32x4 (&kf)[C::kSteps], u32x4 (&vr)[C::kVP]) {
    const char* krow = key_row(a_k, prm.K2, min(blk * 32 + r, Lk - 1)) + g * 16;
#pragma unroll
    for (int s = 0; s < C::kSteps; ++s) kf[s] = *reinterpret_cast<const u32x4*>(krow + s * 32);
#pragma unroll
    for (int i = 0; i < C::kVP / 2; ++i) {
      const int item = lane + i * 64;
      const int pair = item / C::kPPR, col = item % C::kPPR;
      const int j0 = min(blk * 32 + 2 * pair, Lk - 1), j1 = min(blk * 32 + 2 * pair + 1, Lk - 1);
      vr[2 * i] = *reinterpret_cast<const u32x4*>(key_row(a_v, prm.V2, j0) + col * 16);
      vr[2 * i + 1] = *reinterpret_cast<const u32x4*>(key_row(a_v, prm.V2, j1) + col * 16);
    }
  };

  // the first two blocks of this wave are asked for before anything else: their latency covers the query loads
  u32x4 kfa[C::kSteps], vra[C::kVP], kfb[C::kSteps], vrb[C::kVP];
  if (wave < nblk) request(wave, kfa, vra);
  if (wave + NW < nblk) request(wave + NW, kfb, vrb);

  const int q = qt * 32 + r;
  u32x4 qf[C::kSteps];
  {
    const char* qrow = prm.Q.group_row(b, h, prm.q_per_kv, prm.n_resp, min(q, prm.n_q - 1));
#pragma unroll
    for (int s = 0; s < C::kSteps; ++s) qf[s] = *reinterpret_cast<const u32x4*>(qrow + s * 32 + g * 16);
  }
  f32x16 o[C::kDB];
#pragma unroll
  for (int db = 0; db < C::kDB; ++db) o[db] = f32x16{};
  float m = kNegBig, l = 0.f;
  const float c = prm.c;
  uint32_t* vt32 = reinterpret_cast<uint32_t*>(smem + wave * C::kVtBytes);

  auto step = [&](int blk, u32x4 (&kf)[C::kSteps], u32x4 (&vr)[C::kVP]) {
    // V^T of the block into this wave's LDS tile: a 32-bit word holds keys (2*pair, 2*pair+1) of one element.
    // The tile is private to the wave; the fences order this block's stores after the previous block's
    // fragment loads and before this block's.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < C::kVP / 2; ++i) {
      const int item = lane + i * 64;
      const int pair = item / C::kPPR, col = item % C::kPPR;
      const u32x4 a = vr[2 * i], bq = vr[2 * i + 1];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int word = (col * 8 + 2 * w) * (kNarrowVS / 2) + (col / 4) * (kNarrowShift / 4) + pair;
        vt32[word] = (a[w] & 0xFFFFu) | (bq[w] << 16);
        vt32[word + kNarrowVS / 2] = (a[w] >> 16) | (bq[w] & 0xFFFF0000u);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // S^T = K Q^T: keys on rows, queries on columns
    f32x16 s = f32x16{};
#pragma unroll
    for (int st = 0; st < C::kSteps; ++st) mfma_step<T>(kf[st], qf[st], s);
    if (blk + 2 * NW < nblk) request(blk + 2 * NW, kf, vr);
    const int nvalid = Lk - blk * 32;
    if (nvalid < 32) {
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (8 * (i / 4) + 4 * g + (i % 4) >= nvalid) s[i] = -INFINITY;
    }
    // online softmax; lanes l and l^32 hold the same query
    float bm = s[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) bm = fmaxf(bm, s[i]);
    bm = fmaxf(bm, xor32(bm));
    const float cand = bm * c;
    const bool bump = cand > m + kLazyBump;  // the reference is raised lazily, as in the tiled kernel
    if (__any(bump)) {
      const float m_new = bump ? cand : m;
      const float alpha = fast_exp2(m - m_new);
      m = m_new;
      l *= alpha;
#pragma unroll
      for (int db = 0; db < C::kDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
    }
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float pv = fast_exp2(fmaf(s[i], c, -m));
      s[i] = pv;
      psum += pv;
    }
    l += psum;
    // O^T += V^T P^T
#pragma unroll
    for (int tp = 0; tp < 2; ++tp) {
      u32x4 pf;
#pragma unroll
      for (int w = 0; w < 4; ++w) pf[w] = pack_bf16x2(s[8 * tp + 2 * w], s[8 * tp + 2 * w + 1]);
#pragma unroll
      for (int db = 0; db < C::kDB; ++db) {
        const char* rowp =
            reinterpret_cast<const char*>(vt32) + ((db * 32 + r) * kNarrowVS + 16 * tp + 4 * g) * 2 + db * kNarrowShift;
        const u32x2 lo = *reinterpret_cast<const u32x2*>(rowp);
        const u32x2 hi = *reinterpret_cast<const u32x2*>(rowp + 16);
        const u32x4 vf = {lo[0], lo[1], hi[0], hi[1]};
        mfma_step<T>(vf, pf, o[db]);
      }
    }
  };

  for (int blk = wave; blk < nblk; blk += 2 * NW) {
    step(blk, kfa, vra);
    if (blk + NW < nblk) step(blk + NW, kfb, vrb);
  }

  // ---- merge the waves' partial results through LDS (the V tiles are no longer needed)
  const float l_tot = l + xor32(l);
  float* mo = reinterpret_cast<float*>(smem);                          // [wave][db][i][lane]
  float2* ml = reinterpret_cast<float2*>(smem + C::kLds - NW * 32 * 8);  // [wave][query]
  __syncthreads();
#pragma unroll
  for (int db = 0; db < C::kDB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) mo[((wave * C::kDB + db) * 16 + i) * 64 + lane] = o[db][i];
  if (g == 0) ml[wave * 32 + r] = make_float2(m, l_tot);
  __syncthreads();
  float M = kNegBig;
#pragma unroll
  for (int w = 0; w < NW; ++w) M = fmaxf(M, ml[w * 32 + r].x);
  float wgt[NW];
  float L = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const float2 v = ml[w * 32 + r];
    wgt[w] = fast_exp2(v.x - M);
    L += wgt[w] * v.y;
  }
  if (q >= prm.n_q) return;
  const float inv = 1.f / L;
  char* orow = prm.O.group_row(b, h, prm.q_per_kv, prm.n_resp, q);
  // the kDB * 4 groups of four output elements are dealt over the waves
  for (int item = wave; item < C::kDB * 4; item += NW) {
    const int db = item >> 2, qd = item & 3;
    float v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float acc = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) acc += wgt[w] * mo[((w * C::kDB + db) * 16 + 4 * qd + e) * 64 + lane];
      v[e] = acc * inv;
    }
    u32x2 wout;
    wout[0] = pack_bf16x2(v[0], v[1]);
    wout[1] = pack_bf16x2(v[2], v[3]);
    *reinterpret_cast<u32x2*>(orow + (db * 32 + 8 * qd + 4 * g) * 2) = wout;
  }
  if (prm.lse && wave == 0 && g == 0) prm.lse[(int64_t)bh * prm.n_q + q] = (M + __log2f(L)) * kLn2;
}

// Merge the key splits of the query rows: O = sum_s w_s O_s / sum_s w_s l_s, w_s = 2^(m_s - max m).
// A row is served by D/4 consecutive threads (four output elements each, 16-byte loads of the partials).
template <typename T, int D>
__global__ __launch_bounds__(256) void attend_merge_kernel(const AttendParams prm) {
  constexpr int kTPR = D / 4;          // threads per row
  constexpr int kRows = 256 / kTPR;    // rows per workgroup
  const int bh = blockIdx.y;
  const int b = bh / prm.H, h = bh % prm.H;
  const int q = blockIdx.x * kRows + (int)threadIdx.x / kTPR;
  const int e = ((int)threadIdx.x % kTPR) * 4;
  if (q >= prm.n_q) return;
  float M = kNegBig;
  for (int s = 0; s < prm.n_splits; ++s)
    M = fmaxf(M, prm.part_ml[((int64_t)bh * prm.n_splits + s) * prm.n_q + q].x);
  float L = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < prm.n_splits; ++s) {
    const int64_t slot = ((int64_t)bh * prm.n_splits + s) * prm.n_q + q;
    const float2 ml = prm.part_ml[slot];
    const float w = fast_exp2(ml.x - M);
    const float4 v = *reinterpret_cast<const float4*>(prm.part_o + slot * D + e);
    L += w * ml.y;
    acc.x += w * v.x;
    acc.y += w * v.y;
    acc.z += w * v.z;
    acc.w += w * v.w;
  }
  const float inv = 1.f / L;
  char* orow = prm.O.group_row(b, h, prm.q_per_kv, prm.n_resp, q);
  if (sizeof(T) == 2) {
    u32x2 w;
    w[0] = pack_bf16x2(acc.x * inv, acc.y * inv);
    w[1] = pack_bf16x2(acc.z * inv, acc.w * inv);
    *reinterpret_cast<u32x2*>(orow + e * 2) = w;
  } else {
    *reinterpret_cast<float4*>(orow + e * 4) = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
  }
  if (prm.lse && e == 0) prm.lse[(int64_t)bh * prm.n_q + q] = (M + __log2f(L)) * kLn2;
}

// Heads by descending key count, for the compressed call of the tiled kernel: budgets are ragged, the hardware
// hands workgroups to compute units in launch order, and the longest heads should not start last (measured
// on 256 heads with 576...1536 keys: 101 us in this order, 123 us in the given order).  A counting sort by
// 64-key tile count in one workgroup; the order inside a bucket is whatever the atomics give, which does not
// matter: every head's result is independent of when it runs.
constexpr int kOrderThreads = 1024;
constexpr int kOrderBuckets = 1024;

__global__ __launch_bounds__(kOrderThreads) void attend_order_kernel(const int32_t* cu, int64_t capacity, int BH,
                                                                     int n_resp, int32_t* order) {
  __shared__ int count[kOrderBuckets];
  __shared__ int wave_total[kOrderThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  auto bucket_of = [&](int bh) {
    const int64_t c0 = min((int64_t)cu[bh], capacity), c1 = min((int64_t)cu[bh + 1], capacity);
    const int64_t tiles = (c1 - c0 + n_resp + 63) / 64;
    return kOrderBuckets - 1 - (int)min((int64_t)(kOrderBuckets - 1), tiles);  // bucket 0 = longest
  };
  count[tid] = 0;
  __syncthreads();
  for (int bh = tid; bh < BH; bh += kOrderThreads) atomicAdd(&count[bucket_of(bh)], 1);
  __syncthreads();
  // exclusive prefix sum over the buckets, one bucket per thread
  const int mine = count[tid];
  int incl = mine;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int n = __shfl_up(incl, o, 64);
    if (lane >= o) incl += n;
  }
  if (lane == 63) wave_total[wave] = incl;
  __syncthreads();
  int before = 0;
  for (int w = 0; w < wave; ++w) before += wave_total[w];
  count[tid] = before + incl - mine;  // first slot of this bucket
  __syncthreads();
  for (int bh = tid; bh < BH; bh += kOrderThreads) order[atomicAdd(&count[bucket_of(bh)], 1)] = bh;
}

// Queries per workgroup of the tiled kernel for this description.
int tiled_queries(const maskkv_desc* d) {
  return (d->dtype == MASKKV_BF16 && d->d == 64) ? AttCfg<bf16_t, 64>::kQPerBlock : AttCfg<bf16_t, 128>::kQPerBlock;
}

int attend_splits(const maskkv_desc* d, bool full) {
  if (!full) return 1;
  const int64_t qtiles = ((int64_t)d->n_resp * query_heads_per_kv(d) + tiled_queries(d) - 1) / tiled_queries(d);
  const int64_t blocks = qtiles * d->B * d->H;
  int64_t s = (256 + blocks - 1) / blocks;  // one workgroup per compute unit, a single round (measured best)
  const int64_t by_len = ((int64_t)d->P_max + d->n_resp + 511) / 512;
  if (s > by_len) s = by_len;
  if (s > 64) s = 64;
  if (s < 1) s = 1;
  return (int)s;
}

// The narrow kernel is used when the tiled kernel would launch fewer workgroups than there are compute units.
bool attend_is_narrow(const maskkv_desc* d, bool full) {
  if (full || d->dtype != MASKKV_BF16) return false;
  const int64_t qtiles = ((int64_t)d->n_resp * query_heads_per_kv(d) + 127) / 128;
  return qtiles * d->B * d->H < kNarrowBelow;
}

template <int D, int NW>
int launch_attend_narrow(const AttendParams& prm, hipStream_t stream) {
  using C = NarrowCfg<D, NW>;
  static bool raised = false;  // one-time opt-in to more than the default dynamic LDS size
  if (C::kLds > 48 * 1024 && !raised) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attend_narrow_kernel<D, NW>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, C::kLds);
    if (e != hipSuccess) {
      set_error("attend: cannot raise dynamic LDS limit: %s", hipGetErrorString(e));
      (void)hipGetLastError();
      return MASKKV_EHIP;
    }
    raised = true;
  }
  const int nqt = (prm.n_q + 31) / 32;
  const int groups = (prm.BH + 7) / 8 * 8 * nqt;
  hipLaunchKernelGGL((attend_narrow_kernel<D, NW>), dim3(groups), dim3(C::kThreads), C::kLds, stream, prm);
  return check_launch("attend (narrow)");
}

template <typename T, int D>
int launch_attend_t(const AttendParams& prm, int B, hipStream_t stream) {
  using C = AttCfg<T, D>;
  const int64_t qtiles = (prm.n_q + C::kQPerBlock - 1) / C::kQPerBlock;
  const int64_t units = ((int64_t)B * prm.H * prm.n_splits + 7) / 8 * 8;  // (head, split) pairs, whole rounds of XCDs
  if (units * qtiles > 0x7FFFFFFF) {
    set_error("attend: %lld workgroups exceed the launch limit", (long long)(units * qtiles));
    return MASKKV_ESHAPE;
  }
  if (prm.order) {
    hipLaunchKernelGGL(attend_order_kernel, dim3(1), dim3(kOrderThreads), 0, stream, prm.cu, prm.capacity, prm.BH,
                       prm.n_resp, const_cast<int32_t*>(prm.order));
    if (int e = check_launch("attend (order)")) return e;
  }
  static bool raised = false;  // one-time opt-in to more than the default dynamic LDS size
  if (C::kLds > 48 * 1024 && !raised) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attend_kernel<T, D>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, C::kLds);
    if (e != hipSuccess) {
      set_error("attend: cannot raise dynamic LDS limit: %s", hipGetErrorString(e));
      (void)hipGetLastError();
      return MASKKV_EHIP;
    }
    raised = true;
  }
  hipLaunchKernelGGL((attend_kernel<T, D>), dim3((unsigned)(units * qtiles)), dim3(C::kThreads), C::kLds, stream,
                     prm);
  if (int e = check_launch("attend")) return e;
  if (prm.n_splits > 1) {
    constexpr int kRows = 256 / (D / 4);
    hipLaunchKernelGGL((attend_merge_kernel<T, D>), dim3((prm.n_q + kRows - 1) / kRows, B * prm.H), dim3(256), 0,
                       stream, prm);
    return check_launch("attend merge");
  }
  return MASKKV_OK;
}

}  // namespace

size_t attend_workspace_bytes(const maskkv_desc* d, bool full) {
  const int s = attend_splits(d, full);
  if (!full) return attend_is_narrow(d, full) ? 0 : ((size_t)d->B * d->H * sizeof(int32_t) + 255) / 256 * 256;
  if (s == 1) return 0;
  const size_t rows = (size_t)d->B * d->H * s * d->n_resp * query_heads_per_kv(d);
  return (rows * d->d * sizeof(float) + 255) / 256 * 256 + rows * sizeof(float2);
}

int launch_attend(const maskkv_desc* d, const Lens& lens, bool full, const View& Q, const void* Kc, const void* Vc,
                  const int32_t* cu_budget, int64_t capacity, const View& K2, const View& V2, float scale,
                  const View& O, float* lse, void* workspace, hipStream_t stream) {
  AttendParams prm;
  prm.Q = Q;
  prm.K2 = K2;
  prm.V2 = V2;
  prm.O = O;
  prm.lens = lens;
  prm.Kc = reinterpret_cast<const char*>(Kc);
  prm.Vc = reinterpret_cast<const char*>(Vc);
  prm.cu = cu_budget;
  prm.capacity = capacity;
  prm.H = d->H;
  prm.BH = d->B * d->H;
  prm.n_resp = d->n_resp;
  prm.q_per_kv = query_heads_per_kv(d);
  prm.n_q = d->n_resp * prm.q_per_kv;
  prm.full = full ? 1 : 0;
  prm.n_splits = attend_splits(d, full);
  prm.c = scale * kLog2e;
  prm.lse = lse;
  prm.order = (!full && !attend_is_narrow(d, full)) ? reinterpret_cast<const int32_t*>(workspace) : nullptr;
  prm.part_o = nullptr;
  prm.part_ml = nullptr;
  if (prm.n_splits > 1) {
    const size_t rows = (size_t)d->B * d->H * prm.n_splits * prm.n_q;
    prm.part_o = reinterpret_cast<float*>(workspace);
    prm.part_ml = reinterpret_cast<float2*>(reinterpret_cast<char*>(workspace) +
                                            (rows * d->d * sizeof(float) + 255) / 256 * 256);
  }
  if (attend_is_narrow(d, full))  // (eight waves per 32-query tile measured slower: 20.6 vs 17.6 us at the 32k prompt)
    return d->d == 128 ? launch_attend_narrow<128, 4>(prm, stream) : launch_attend_narrow<64, 4>(prm, stream);
  if (d->dtype == MASKKV_BF16)
    return d->d == 128 ? launch_attend_t<bf16_t, 128>(prm, d->B, stream) : launch_attend_t<bf16_t, 64>(prm, d->B, stream);
  return d->d == 128 ? launch_attend_t<float, 128>(prm, d->B, stream) : launch_attend_t<float, 64>(prm, d->B, stream);
}

}  // namespace maskkv
