// Eviction as a row gather (MaskKV appendix "Prompt-state Exclusion": the cache keeps prompt K/V only,
// and of those only the selected rows).  Every thread moves one 16-byte piece of a K row and of the
// matching V row; a row's pieces are handled by consecutive lanes, so reads and writes are coalesced
// per row and the packed destination is written as one contiguous stream.
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

__global__ __launch_bounds__(256) void compact_kernel(const CompactParams prm) {
  const int ppr = prm.row_bytes / 16;  // pieces per row
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = gid / ppr;
  const int piece = (int)(gid % ppr);
  const int64_t total = min((int64_t)prm.cu[prm.BH], prm.capacity);
  if (row >= total) return;
  // head of this row: largest bh with cu[bh] <= row
  int lo = 0, hi = prm.BH;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)prm.cu[mid] <= row) lo = mid; else hi = mid;
  }
  const int b = lo / prm.H;
  const int h = lo % prm.H;
  // a caller-supplied index outside the prompt is clamped rather than read out of bounds
  const int src = min(max(prm.idx[row], 0), max(prm.lens.P[b] - 1, 0));
  const u32x4 kv = *reinterpret_cast<const u32x4*>(prm.K.row(b, h, src) + piece * 16);
  const u32x4 vv = *reinterpret_cast<const u32x4*>(prm.V.row(b, h, src) + piece * 16);
  *reinterpret_cast<u32x4*>(prm.Kc + row * prm.row_bytes + piece * 16) = kv;
  *reinterpret_cast<u32x4*>(prm.Vc + row * prm.row_bytes + piece * 16) = vv;
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
  const int64_t threads = capacity * (prm.row_bytes / 16);
  const int64_t blocks = (threads + 255) / 256;
  hipLaunchKernelGGL(compact_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, prm);
  return check_launch("compact");
}

}  // namespace maskkv
