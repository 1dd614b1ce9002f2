// Eviction as a row gather (MaskKV appendix "Prompt-state Exclusion": the cache keeps prompt K/V only,
// and of those only the selected rows).  Every thread moves one 16-byte piece of two K rows and of the
// matching V rows (four independent 16-byte loads in flight per lane); a row's pieces are handled by
// consecutive lanes, so reads and writes are coalesced per row and the packed destination is written as one
// contiguous stream.  The head that owns a destination row is found from the prefix sums cu: one wave
// searches them 64 ways at a time for the workgroup's first row (two dependent loads for up to 4096
// heads), and every thread walks on from there (rows of one workgroup rarely span more than two heads).
#include "kernels.hpp"

namespace maskkv {

namespace {

struct CompactParams {
  View K, V;
  Lens lens;
  int H, BH;
  int row_bytes;
  const int32_t* idx;
  const int32_t* cu;
  int64_t capacity;
  char* Kc;
  char* Vc;
};

constexpr int kCmpRows = 2;  // destination rows per thread

__global__ __launch_bounds__(256) void compact_kernel(const CompactParams prm) {
  __shared__ int first_head;
  const int ppr = prm.row_bytes / 16;  // pieces per row: 8, 16 or 32
  const int rows_per_pass = 256 / ppr;
  const int64_t row0 = (int64_t)blockIdx.x * rows_per_pass * kCmpRows;
  const int64_t total = min((int64_t)prm.cu[prm.BH], prm.capacity);
  if (row0 >= total) return;
  if (threadIdx.x < 64) {
    // largest head lo with cu[lo] <= row0; invariant cu[lo] <= row0 < cu[hi]
    const int lane = threadIdx.x;
    int lo = 0, hi = prm.BH;
    while (hi - lo > 1) {
      const int step = (hi - lo + 63) / 64;
      const int probe = min(lo + (lane + 1) * step, hi);
      const int nle = __popcll(__ballot((int64_t)prm.cu[probe] <= row0));  // true for a prefix of the lanes
      const int new_lo = nle == 0 ? lo : min(lo + nle * step, hi);
      hi = nle == 64 ? hi : min(lo + (nle + 1) * step, hi);
      lo = new_lo;
    }
    if (lane == 0) first_head = lo;
  }
  __syncthreads();

  const int piece = threadIdx.x % ppr;
  int64_t row[kCmpRows];
  const char* ksrc[kCmpRows];
  const char* vsrc[kCmpRows];
  bool live[kCmpRows];
#pragma unroll
  for (int u = 0; u < kCmpRows; ++u) {
    row[u] = row0 + u * rows_per_pass + threadIdx.x / ppr;
    live[u] = row[u] < total;
    const int64_t rr = live[u] ? row[u] : row0;
    int bh = first_head;
    while (bh + 1 < prm.BH && (int64_t)prm.cu[bh + 1] <= rr) ++bh;
    const int b = bh / prm.H;
    const int h = bh % prm.H;
    // a caller-supplied index outside the prompt is clamped rather than read out of bounds
    const int src = min(max(prm.idx[rr], 0), max(prm.lens.P[b] - 1, 0));
    ksrc[u] = prm.K.row(b, h, src) + piece * 16;
    vsrc[u] = prm.V.row(b, h, src) + piece * 16;
  }
  u32x4 kv[kCmpRows], vv[kCmpRows];
#pragma unroll
  for (int u = 0; u < kCmpRows; ++u) {
    kv[u] = *reinterpret_cast<const u32x4*>(ksrc[u]);
    vv[u] = *reinterpret_cast<const u32x4*>(vsrc[u]);
  }
#pragma unroll
  for (int u = 0; u < kCmpRows; ++u) {
    if (live[u]) {
      *reinterpret_cast<u32x4*>(prm.Kc + row[u] * prm.row_bytes + piece * 16) = kv[u];
      *reinterpret_cast<u32x4*>(prm.Vc + row[u] * prm.row_bytes + piece * 16) = vv[u];
    }
  }
}

}  // namespace

int launch_compact(const maskkv_desc* d, const Lens& lens, const View& K, const View& V, const int32_t* idx, const int32_t* cu_budget,
                   int64_t capacity, void* Kc, void* Vc, hipStream_t stream) {
  if (capacity == 0) return MASKKV_OK;
  CompactParams prm;
  prm.K = K;
  prm.V = V;
  prm.lens = lens;
  prm.H = d->H;
  prm.BH = d->B * d->H;
  prm.row_bytes = d->d * (d->dtype == MASKKV_BF16 ? 2 : 4);
  prm.idx = idx;
  prm.cu = cu_budget;
  prm.capacity = capacity;
  prm.Kc = reinterpret_cast<char*>(Kc);
  prm.Vc = reinterpret_cast<char*>(Vc);
  const int64_t rows_per_block = (256 / (prm.row_bytes / 16)) * kCmpRows;
  const int64_t blocks = (capacity + rows_per_block - 1) / rows_per_block;
  hipLaunchKernelGGL(compact_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, prm);
  return check_launch("compact");
}

}  // namespace maskkv
