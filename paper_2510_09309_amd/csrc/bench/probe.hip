// Measurement library (libmaskkv_bench.so): not part of the method and not part of libmaskkv.so.
//   maskkv_bench_probe         kernels that each exercise one resource of the chip, so that a harness can quote
//                              kernel rates against what this machine sustains at the clock it actually runs at;
//   maskkv_bench_score_marked  maskkv_score with HIP events recorded at its stage boundaries (it calls the body
//                              of maskkv_score inside libmaskkv.so).
#include <stdio.h>

#include "../kernels.hpp"
#include "../../../include/maskkv_bench.h"

namespace maskkv {

namespace {

constexpr int kProbeThreads = 256;
constexpr int kMfmaChains = 4;  // independent accumulators per wave (an MFMA's result is needed 32 cycles later)
constexpr int kExpChains = 8;

// Every wave issues iters * kMfmaChains v_mfma_f32_32x32x16_bf16 from registers only, all with the same
// (constant) operands: the data-sheet situation.
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

// The matrix-pipe stream of the scoring and attention kernels, from registers only: chains of eight MFMAs (one
// 32 x 32 logits block at head_dim 128) that start from zero, alternating between two accumulators, the A operand
// taken from 16 and the B operand from 8 different register sets that are loaded from `src` (the caller fills it
// with the bit patterns the kernels really see, e.g. Gaussian bf16).  The matrix pipe draws power by the bits it
// toggles: this is the rate it sustains on such data, which is what a kernel can be held against.
__global__ __launch_bounds__(kProbeThreads) void probe_mfma_data_kernel(int iters, const u32x4* src, float* out) {
  u32x4 ka[2][8], qf[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    ka[0][i] = src[(threadIdx.x & 63) + 64 * i];
    ka[1][i] = src[(threadIdx.x & 63) + 64 * (8 + i)];
    qf[i] = src[(threadIdx.x & 63) + 64 * (16 + i)];
  }
  f32x16 acc[2] = {f32x16{}, f32x16{}};
  float s = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      s += acc[kb][0];  // the previous block is consumed before it is overwritten
      acc[kb] = f32x16{};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) mfma_step<bf16_t>(ka[kb][ks], qf[ks], acc[kb]);
    }
  }
#pragma unroll
  for (int u = 0; u < 2; ++u)
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

// The scoring kernels' form-and-reduce pipeline from registers only, on data: per iteration every wave forms the
// logits of two 32x32 blocks (16 MFMAs at head_dim 128, two chains of eight that start from zero, operands from the
// 24 register sets loaded from `src`) into one accumulator pair while it takes the exponentials of the pair formed
// one iteration earlier (32 x (multiply, v_exp_f32, add) per lane), in one basic block, as the kernels do.  Unlike
// probe_mix_kernel the vector work consumes the matrix pipe's results and the operands toggle like real data.
__global__ __launch_bounds__(kProbeThreads) void probe_pipeline_kernel(int iters, const u32x4* src, float* out) {
  u32x4 ka[2][8], qf[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    ka[0][i] = src[(threadIdx.x & 63) + 64 * i];
    ka[1][i] = src[(threadIdx.x & 63) + 64 * (8 + i)];
    qf[i] = src[(threadIdx.x & 63) + 64 * (16 + i)];
  }
  f32x16 accA[2] = {f32x16{}, f32x16{}}, accB[2] = {f32x16{}, f32x16{}};
  const float c = 0.127f;
  float sum = 0.f;
  // `flip` pairs the operand sets differently in the two stages of a loop trip and one operand word changes from
  // trip to trip, so that no block is the same computation as another one.
  auto stage = [&](f32x16 (&next)[2], f32x16 (&cur)[2], int flip) {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) next[blk] = f32x16{};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) mfma_step<bf16_t>(ka[blk ^ flip][ks], qf[(ks + flip) & 7], next[blk]);
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int i = 0; i < 16; ++i) sum += fast_exp2(cur[blk][i] * c);
  };
  for (int it = 0; it < iters; it += 2) {
    qf[0][0] ^= 0x00010000u;  // the lowest mantissa bit of one bf16 operand element
    stage(accB, accA, 0);
    stage(accA, accB, 1);
  }
  float s = sum;
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += accA[u][i] + accB[u][i];
  out[(int64_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

// Do the matrix pipe and the vector pipe of a SIMD work at the same time for different waves?  Workgroups of eight
// waves (waves w and w + 4 share a SIMD): per iteration waves 0-3 issue the sixteen MFMAs of probe_mfma_data_kernel,
// waves 4-7 the 32 x (multiply, v_exp_f32, add) of a logits block pair.  WHO = 0: both halves work, 1: the matrix
// half alone (the other half exits at once), 2: the vector half alone.
constexpr int kSplitThreads = 512;

template <int WHO>
__global__ __launch_bounds__(kSplitThreads) void probe_split_kernel(int iters, const u32x4* src, float* out) {
  const int lane = threadIdx.x & 63;
  const bool vector_half = threadIdx.x >= kSplitThreads / 2;
  float s = 0.f;
  if (!vector_half) {
    if (WHO == 2) return;
    u32x4 ka[8], qf[8];  // (sixteen operand sets: a 512-thread workgroup leaves a wave 128 registers)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      ka[i] = src[lane + 64 * i];
      qf[i] = src[lane + 64 * (16 + i)];
    }
    f32x16 acc[2] = {f32x16{}, f32x16{}};
    for (int it = 0; it < iters; it += 2) {
      qf[0][0] ^= 0x00010000u;  // the lowest mantissa bit of one bf16 operand element
#pragma unroll
      for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
#pragma unroll
          for (int blk = 0; blk < 2; ++blk) mfma_step<bf16_t>(ka[(ks + blk + half) & 7], qf[ks], acc[blk]);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 16; ++i) s += acc[u][i];
  } else {
    if (WHO == 1) return;
    float x[32], sum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 32; ++u) x[u] = 0.01f * (float)(lane + u + 1);
    const float c = 0.127f;
    for (int it = 0; it < iters; it += 2) {
#pragma unroll
      for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int u = 0; u < 32; ++u) {
          x[u] = fast_exp2(x[u] * c);
          sum[u & 3] += x[u];
        }
    }
    s = (sum[0] + sum[1]) + (sum[2] + sum[3]);
  }
  out[(int64_t)blockIdx.x * kSplitThreads + threadIdx.x] = s;
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

thread_local char g_bench_err[256] = "";

int fail(const char* msg) {
  snprintf(g_bench_err, sizeof(g_bench_err), "%s", msg);
  return MASKKV_EINVAL;
}

int launched(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return MASKKV_OK;
  snprintf(g_bench_err, sizeof(g_bench_err), "%s: %s", what, hipGetErrorString(e));
  return MASKKV_EHIP;
}

}  // namespace
}  // namespace maskkv

using namespace maskkv;

extern "C" {

const char* maskkv_bench_last_error(void) { return g_bench_err; }

int maskkv_bench_probe(int which, int32_t iters, const void* src, void* dst, int64_t bytes, int64_t dst_bytes,
                       int32_t groups, void* stream_, double* work) {
  hipStream_t stream = reinterpret_cast<hipStream_t>(stream_);
  if (which < 0 || which > 9 || !dst || groups < 1 || groups > (1 << 20))
    return fail("probe: which outside 0..9, dst NULL or groups outside 1..2^20");
  if (which != 2 && dst_bytes < (int64_t)groups * (which >= 7 ? kSplitThreads : kProbeThreads) * 4)
    return fail("probe: dst is smaller than one word per launched thread");
  const bool arithmetic = which == 0 || which == 1 || which >= 4;
  if (arithmetic && iters < 1) return fail("probe: iters < 1");
  if (which >= 5 && (!src || ((uintptr_t)src & 15) || bytes < 64 * 24 * 16))
    return fail("probe: the data-fed matrix probe reads 24 KiB of operands from a 16-byte aligned src");
  if ((which == 2 || which == 3) &&
      (!src || bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15) ||
       (which == 2 && dst_bytes < bytes)))
    return fail("probe: streaming needs 16-byte aligned src and dst, a positive multiple of 16 bytes, and room in dst");
  if (work) {
    const double waves = (double)groups * (kProbeThreads / 64);
    switch (which) {
      case 0: *work = waves * kMfmaChains * iters * 32768.0; break;  // 2*32*32*16 flop per MFMA
      case 1: *work = (double)groups * kProbeThreads * kExpChains * iters; break;
      case 2: *work = 2.0 * (double)bytes; break;
      case 3: *work = (double)bytes; break;
      case 6: *work = waves * 16.0 * ((iters + 1) / 2 * 2) * 32768.0; break;  // (iterations come in pairs)
      case 7:  // (iterations come in pairs)
      case 8: *work = (double)groups * 4 * 16.0 * ((iters + 1) / 2 * 2) * 32768.0; break;  // four matrix waves per workgroup
      case 9: *work = (double)groups * 256 * 32.0 * ((iters + 1) / 2 * 2); break;  // exponentials of the vector half
      default: *work = waves * 16.0 * iters * 32768.0; break;  // 4, 5: sixteen MFMAs per iteration
    }
  }
  float* out = reinterpret_cast<float*>(dst);
  switch (which) {
    case 0:
      hipLaunchKernelGGL(probe_mfma_kernel, dim3(groups), dim3(kProbeThreads), 0, stream, iters, out);
      return launched("probe (mfma)");
    case 1:
      hipLaunchKernelGGL(probe_exp_kernel, dim3(groups), dim3(kProbeThreads), 0, stream, iters, out);
      return launched("probe (exp)");
    case 2:
      hipLaunchKernelGGL(probe_copy_kernel, dim3(groups), dim3(kProbeThreads), 0, stream,
                         reinterpret_cast<const u32x4*>(src), reinterpret_cast<u32x4*>(dst), bytes / 16);
      return launched("probe (copy)");
    case 3:
      hipLaunchKernelGGL(probe_read_kernel, dim3(groups), dim3(kProbeThreads), 0, stream,
                         reinterpret_cast<const u32x4*>(src), reinterpret_cast<uint32_t*>(dst), bytes / 16);
      return launched("probe (read)");
    case 4:
      hipLaunchKernelGGL(probe_mix_kernel, dim3(groups), dim3(kProbeThreads), 0, stream, iters, out);
      return launched("probe (mix)");
    case 5:
      hipLaunchKernelGGL(probe_mfma_data_kernel, dim3(groups), dim3(kProbeThreads), 0, stream, iters,
                         reinterpret_cast<const u32x4*>(src), out);
      return launched("probe (mfma on data)");
    case 7:
      hipLaunchKernelGGL(probe_split_kernel<0>, dim3(groups), dim3(kSplitThreads), 0, stream, iters,
                         reinterpret_cast<const u32x4*>(src), out);
      return launched("probe (matrix waves and vector waves)");
    case 8:
      hipLaunchKernelGGL(probe_split_kernel<1>, dim3(groups), dim3(kSplitThreads), 0, stream, iters,
                         reinterpret_cast<const u32x4*>(src), out);
      return launched("probe (matrix waves alone)");
    case 9:
      hipLaunchKernelGGL(probe_split_kernel<2>, dim3(groups), dim3(kSplitThreads), 0, stream, iters,
                         reinterpret_cast<const u32x4*>(src), out);
      return launched("probe (vector waves alone)");
    default:
      hipLaunchKernelGGL(probe_pipeline_kernel, dim3(groups), dim3(kProbeThreads), 0, stream, iters,
                         reinterpret_cast<const u32x4*>(src), out);
      return launched("probe (form-and-reduce pipeline on data)");
  }
}

int maskkv_bench_score_marked(const maskkv_desc* desc, const maskkv_tensor* Q_mask, const maskkv_tensor* K_full,
                              float scale, float* scores, int64_t score_stride, float* prompt_mass, void* workspace,
                              size_t workspace_bytes, void* stream, void* const* events) {
  return score_entry(desc, Q_mask, K_full, scale, scores, score_stride, prompt_mass, workspace, workspace_bytes, stream,
                     events);
}

}  // extern "C"
