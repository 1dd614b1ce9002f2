// Measurement probes: what this chip sustains on the three resources that bound the MaskKV kernels - the
// bf16 matrix pipe, the v_exp_f32 rate of the vector pipe, and HBM streaming (copy and read-only).  They are not part of the
// method; the benchmark runs them next to the kernels so that every roofline fraction can also be quoted
// against a rate measured on the same box at the clock it actually runs at.
#include "kernels.hpp"

namespace maskkv {

namespace {

constexpr int kProbeThreads = 256;
constexpr int kMfmaChains = 4;  // independent accumulators per wave (an MFMA's result is needed 32 cycles later)
constexpr int kExpChains = 8;

// Every wave issues iters * kMfmaChains v_mfma_f32_32x32x16_bf16 from registers only.
__global__ __launch_bounds__(kProbeThreads) void probe_mfma_kernel(int iters, float* out) {
  const uint32_t seed = 0x3C003C00u + (threadIdx.x & 7u);  // two small positive bf16 values per word
  const u32x4 a = {seed, seed + 1u, seed + 2u, seed + 3u};
  const u32x4 b = {seed + 4u, seed + 5u, seed + 6u, seed + 7u};
  f32x16 acc[kMfmaChains];
#pragma unroll
  for (int u = 0; u < kMfmaChains; ++u) acc[u] = f32x16{};
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int u = 0; u < kMfmaChains; ++u) mfma_step<bf16_t>(a, b, acc[u]);
  }
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < kMfmaChains; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[u][i];
  out[(int64_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

// The instruction mix of the scoring kernels from registers only: per iteration every wave issues 16 MFMAs (the
// logits of two 32x32 blocks at head_dim 128) and, per lane, 32 x (fma, v_exp_f32, add) (their exponentials and
// sums), as independent streams in one basic block.  What this sustains bounds a scoring pass from above: no
// tile staging, no barriers, no memory.
__global__ __launch_bounds__(kProbeThreads) void probe_mix_kernel(int iters, float* out) {
  const uint32_t seed = 0x3C003C00u + (threadIdx.x & 7u);
  const u32x4 a = {seed, seed + 1u, seed + 2u, seed + 3u};
  const u32x4 b = {seed + 4u, seed + 5u, seed + 6u, seed + 7u};
  f32x16 acc[kMfmaChains];
#pragma unroll
  for (int u = 0; u < kMfmaChains; ++u) acc[u] = f32x16{};
  float x[32], sum = 0.f;
#pragma unroll
  for (int u = 0; u < 32; ++u) x[u] = 0.01f * (float)(threadIdx.x + u + 1);
  const float c = 0.127f;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int u = 0; u < kMfmaChains; ++u) mfma_step<bf16_t>(a, b, acc[u]);
#pragma unroll
    for (int u = 0; u < 32; ++u) {
      x[u] = fast_exp2(fmaf(x[u], c, -1.0f));
      sum += x[u];
    }
  }
  float s = sum;
#pragma unroll
  for (int u = 0; u < kMfmaChains; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[u][i];
  out[(int64_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

// Every lane runs iters * kExpChains v_exp_f32 (x <- 2^-|x|: the sign and magnitude modifiers are free, the
// values stay in (0, 1]).
__global__ __launch_bounds__(kProbeThreads) void probe_exp_kernel(int iters, float* out) {
  float x[kExpChains];
#pragma unroll
  for (int u = 0; u < kExpChains; ++u) x[u] = 0.01f * (float)(threadIdx.x + u + 1);
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int u = 0; u < kExpChains; ++u) x[u] = fast_exp2(-__builtin_fabsf(x[u]));
  }
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < kExpChains; ++u) s += x[u];
  out[(int64_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

// Streaming copy, 16 bytes per lane, four independent loads in flight.
__global__ __launch_bounds__(kProbeThreads) void probe_copy_kernel(const u32x4* src, u32x4* dst, int64_t pieces) {
  const int64_t stride = (int64_t)gridDim.x * kProbeThreads;
  int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
  for (; i + 3 * stride < pieces; i += 4 * stride) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * stride);
  }
  for (; i < pieces; i += stride) dst[i] = src[i];
}

// Streaming read, 16 bytes per lane, eight independent loads in flight; the words are folded into one value
// per thread so that the loads cannot be dropped.
__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const u32x4* src, uint32_t* out, int64_t pieces) {
  const int64_t stride = (int64_t)gridDim.x * kProbeThreads;
  int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
  uint32_t acc = 0u;
  for (; i + 7 * stride < pieces; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
  }
  for (; i < pieces; i += stride) {
    const u32x4 v = src[i];
    acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  out[(int64_t)blockIdx.x * kProbeThreads + threadIdx.x] = acc;
}

}  // namespace

int launch_probe(int which, int iters, const void* src, void* dst, int64_t bytes, int groups, hipStream_t stream) {
  if (which == 0) {
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(groups), dim3(kProbeThreads), 0, stream, iters,
                       reinterpret_cast<float*>(dst));
    return check_launch("probe (mfma)");
  }
  if (which == 1) {
    hipLaunchKernelGGL(probe_exp_kernel, dim3(groups), dim3(kProbeThreads), 0, stream, iters,
                       reinterpret_cast<float*>(dst));
    return check_launch("probe (exp)");
  }
  if (which == 4) {
    hipLaunchKernelGGL(probe_mix_kernel, dim3(groups), dim3(kProbeThreads), 0, stream, iters,
                       reinterpret_cast<float*>(dst));
    return check_launch("probe (mix)");
  }
  if (which == 3) {
    hipLaunchKernelGGL(probe_read_kernel, dim3(groups), dim3(kProbeThreads), 0, stream,
                       reinterpret_cast<const u32x4*>(src), reinterpret_cast<uint32_t*>(dst), bytes / 16);
    return check_launch("probe (read)");
  }
  hipLaunchKernelGGL(probe_copy_kernel, dim3(groups), dim3(kProbeThreads), 0, stream,
                     reinterpret_cast<const u32x4*>(src), reinterpret_cast<u32x4*>(dst), bytes / 16);
  return check_launch("probe (copy)");
}

}  // namespace maskkv
