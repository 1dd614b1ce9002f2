// Layer importance (MaskKV Section 3.3, Stage 2, layer level):
//   I = 1 - mean_i cos_sim(h_in[i, :], h_out[i, :])
// over the n token rows of a layer's attention sub-layer input and output hidden states.
//
// Pure streaming reduction (two rows of `hidden` elements read per token, three dot products): HBM-bound.
// One wave takes one token row at a time: every lane reads 16-byte pieces of both rows, the three sums
// are reduced across the wave, and the wave keeps a running sum of cosines.  Rows are dealt to the waves of
// the grid round-robin, each workgroup writes one partial sum, and a second one-workgroup kernel adds the
// partials in a fixed order (the result is deterministic).
//
// The same row-wise cosine serves the response-token refresh criterion of the dLLM-Cache background
// (Section 3.1): S_shift = { i : cos_sim(V_i at step t, V_i at step t-1) < delta }.  There the per-row
// cosines are written out and a one-workgroup kernel turns them into the ascending list of positions.
#include "kernels.hpp"

namespace maskkv {

namespace {

constexpr int kImpThreads = 256;
constexpr int kImpWaves = kImpThreads / 64;
constexpr int kImpGroups = 2048;  // eight resident workgroups per compute unit
constexpr int kImpUnroll = 8;

struct ImportanceParams {
  const char* h_in;
  const char* h_out;
  int64_t n, row_bytes;
  int hidden;
  float* partial;     // [kImpGroups]
  float* importance;  // [1]
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename T>
__device__ __forceinline__ void accumulate(const u32x4& a, const u32x4& b, float& dot, float& na, float& nb) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const uint32_t ua = a[w], ub = b[w];
    if (sizeof(T) == 2) {  // two bf16 per word: a bf16 is the upper half of the fp32 with the same value
      const float a0 = as_f32(ua << 16), a1 = as_f32(ua & 0xFFFF0000u);
      const float b0 = as_f32(ub << 16), b1 = as_f32(ub & 0xFFFF0000u);
      dot = fmaf(a0, b0, fmaf(a1, b1, dot));
      na = fmaf(a0, a0, fmaf(a1, a1, na));
      nb = fmaf(b0, b0, fmaf(b1, b1, nb));
    } else {
      const float a0 = as_f32(ua), b0 = as_f32(ub);
      dot = fmaf(a0, b0, dot);
      na = fmaf(a0, a0, na);
      nb = fmaf(b0, b0, nb);
    }
  }
}

// Cosine similarity of two rows of `pieces` 16-byte pieces, computed by one wave; every lane returns it.
template <typename T>
__device__ __forceinline__ float row_cosine(const char* a, const char* b, int pieces, int lane) {
  float dot = 0.f, na = 0.f, nb = 0.f;
  int p = lane;
  for (; p + (kImpUnroll - 1) * 64 < pieces; p += kImpUnroll * 64) {  // 2 * kImpUnroll independent 16-byte loads
    u32x4 va[kImpUnroll], vb[kImpUnroll];                             // in flight per lane; the data is read once
#pragma unroll
    for (int u = 0; u < kImpUnroll; ++u) {
      va[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(a + (int64_t)(p + u * 64) * 16));
      vb[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(b + (int64_t)(p + u * 64) * 16));
    }
#pragma unroll
    for (int u = 0; u < kImpUnroll; ++u) accumulate<T>(va[u], vb[u], dot, na, nb);
  }
  for (; p < pieces; p += 64)
    accumulate<T>(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(a + (int64_t)p * 16)),
                  __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(b + (int64_t)p * 16)), dot, na, nb);
  dot = wave_sum(dot);
  na = wave_sum(na);
  nb = wave_sum(nb);
  return dot / (sqrtf(na) * sqrtf(nb));
}

template <typename T>
__global__ __launch_bounds__(kImpThreads) void importance_kernel(const ImportanceParams prm) {
  __shared__ float wsum[kImpWaves];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int pieces = prm.hidden * (int)sizeof(T) / 16;  // 16-byte pieces per row
  float cos_sum = 0.f;
  for (int64_t row = (int64_t)blockIdx.x * kImpWaves + wave; row < prm.n; row += (int64_t)gridDim.x * kImpWaves)
    cos_sum += row_cosine<T>(prm.h_in + row * prm.row_bytes, prm.h_out + row * prm.row_bytes, pieces, lane);
  if (lane == 0) wsum[wave] = cos_sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int w = 0; w < kImpWaves; ++w) s += wsum[w];
    prm.partial[blockIdx.x] = s;
  }
}

__global__ __launch_bounds__(256) void importance_finish_kernel(const ImportanceParams prm, int groups) {
  __shared__ float red[256];
  float s = 0.f;
  for (int i = threadIdx.x; i < groups; i += 256) s += prm.partial[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) prm.importance[0] = 1.f - red[0] / (float)prm.n;
}

// ---- value shift: per-row cosines, then the ascending list of rows below the threshold -------------------
struct ShiftParams {
  const char* v_now;
  const char* v_prev;
  int64_t n, row_bytes;
  int width;
  float delta;
  float* cos;        // [n]
  int32_t* refresh;  // [n]
  int32_t* count;    // [1]
};

template <typename T>
__global__ __launch_bounds__(kImpThreads) void shift_cos_kernel(const ShiftParams prm) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int pieces = prm.width * (int)sizeof(T) / 16;
  for (int64_t row = (int64_t)blockIdx.x * kImpWaves + wave; row < prm.n; row += (int64_t)gridDim.x * kImpWaves) {
    const float c = row_cosine<T>(prm.v_now + row * prm.row_bytes, prm.v_prev + row * prm.row_bytes, pieces, lane);
    if (lane == 0) prm.cos[row] = c;
  }
}

constexpr int kCollectThreads = 1024;

// One workgroup walks the cosines 1024 at a time and appends the positions below the threshold in order:
// a ballot ranks the flagged lanes inside each wave, the wave totals are prefix-summed through LDS.
__global__ __launch_bounds__(kCollectThreads) void shift_collect_kernel(const ShiftParams prm) {
  constexpr int kWaves = kCollectThreads / 64;
  __shared__ int wave_total[kWaves];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  int64_t written = 0;
  for (int64_t base = 0; base < prm.n; base += kCollectThreads) {
    const int64_t i = base + threadIdx.x;
    const bool flag = i < prm.n && prm.cos[i] < prm.delta;
    const uint64_t mask = __ballot(flag);
    const int rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
    if (lane == 0) wave_total[wave] = __popcll(mask);
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const int t = wave_total[w];
      before += w < wave ? t : 0;
      all += t;
    }
    if (flag) prm.refresh[written + before + rank] = (int32_t)i;
    written += all;
    __syncthreads();
  }
  if (threadIdx.x == 0) prm.count[0] = (int32_t)written;
}

}  // namespace

int launch_value_shift(const void* v_now, const void* v_prev, int64_t n, int width, int dtype, int64_t row_bytes,
                       float delta, float* cos, int32_t* refresh, int32_t* count, hipStream_t stream) {
  ShiftParams prm;
  prm.v_now = reinterpret_cast<const char*>(v_now);
  prm.v_prev = reinterpret_cast<const char*>(v_prev);
  prm.n = n;
  prm.row_bytes = row_bytes;
  prm.width = width;
  prm.delta = delta;
  prm.cos = cos;
  prm.refresh = refresh;
  prm.count = count;
  const int64_t want = (n + kImpWaves - 1) / kImpWaves;
  const int groups = (int)(want < kImpGroups ? want : kImpGroups);
  if (dtype == MASKKV_BF16)
    hipLaunchKernelGGL(shift_cos_kernel<bf16_t>, dim3(groups), dim3(kImpThreads), 0, stream, prm);
  else
    hipLaunchKernelGGL(shift_cos_kernel<float>, dim3(groups), dim3(kImpThreads), 0, stream, prm);
  if (int e = check_launch("value shift")) return e;
  hipLaunchKernelGGL(shift_collect_kernel, dim3(1), dim3(kCollectThreads), 0, stream, prm);
  return check_launch("value shift (collect)");
}

size_t layer_importance_workspace_bytes() { return kImpGroups * sizeof(float); }

int launch_layer_importance(const void* h_in, const void* h_out, int64_t n, int hidden, int dtype, int64_t row_bytes,
                            float* importance, void* workspace, hipStream_t stream) {
  ImportanceParams prm;
  prm.h_in = reinterpret_cast<const char*>(h_in);
  prm.h_out = reinterpret_cast<const char*>(h_out);
  prm.n = n;
  prm.row_bytes = row_bytes;
  prm.hidden = hidden;
  prm.partial = reinterpret_cast<float*>(workspace);
  prm.importance = importance;
  const int64_t want = (n + kImpWaves - 1) / kImpWaves;
  const int groups = (int)(want < kImpGroups ? want : kImpGroups);
  if (dtype == MASKKV_BF16)
    hipLaunchKernelGGL(importance_kernel<bf16_t>, dim3(groups), dim3(kImpThreads), 0, stream, prm);
  else
    hipLaunchKernelGGL(importance_kernel<float>, dim3(groups), dim3(kImpThreads), 0, stream, prm);
  if (int e = check_launch("layer importance")) return e;
  hipLaunchKernelGGL(importance_finish_kernel, dim3(1), dim3(256), 0, stream, prm, groups);
  return check_launch("layer importance (finish)");
}

}  // namespace maskkv
