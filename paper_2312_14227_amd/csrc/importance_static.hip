// Eq. 2 importance reduction for callers that cannot allocate device memory (code under HIP graph
// capture, serving loops, harnesses that forbid hipMalloc): the same two reduction kernels as
// et_importance, with the chunk table, the chunk sums and the per-tensor offsets kept in a
// file-scope device array instead of the caller's workspace.  No hipMalloc, no hipFree, no copy
// from host memory: the chunk table is written by a small kernel from its launch arguments.
//
// Every call on one GPU uses that GPU's copy of the array and overwrites what the previous call
// left there; nothing in it has to start at zero (every entry that is read has been written by the
// same call).  Calls that overlap on one GPU (two streams, two threads) race.
#include <mutex>

#include "context.h"
#include "et.h"
#include "kernels.h"

namespace {

using et::TensorSeg;
using et_exec::SEG_ELEMS;

constexpr uint32_t MAX_STATIC_TENSORS = ET_STATIC_MAX_TENSORS;
constexpr uint32_t MAX_STATIC_SEGS = ET_STATIC_MAX_CHUNKS;
constexpr int MAX_DEVICES = 64;

// layout of the array (all offsets multiples of 256 bytes)
constexpr size_t OFF_SEGS = 0;                                                          // TensorSeg [MAX_STATIC_SEGS]
constexpr size_t OFF_PARTIAL = OFF_SEGS + sizeof(TensorSeg) * MAX_STATIC_SEGS;           // double [MAX_STATIC_SEGS]
constexpr size_t OFF_BEGIN = OFF_PARTIAL + sizeof(double) * MAX_STATIC_SEGS;             // uint32 [MAX_STATIC_TENSORS + 1]
constexpr size_t SCRATCH_BYTES = ((OFF_BEGIN + sizeof(uint32_t) * (MAX_STATIC_TENSORS + 1) + 255) / 256) * 256;
static_assert(OFF_PARTIAL % 256 == 0 && OFF_BEGIN % 256 == 0, "pieces of the scratch array are 256-byte aligned");

// In host code this name is only a handle for hipGetSymbolAddress: the device address is looked up
// once per device and everything below uses that address.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

std::mutex g_lock;
unsigned char* g_scratch_ptr[MAX_DEVICES];   // per device: where that GPU keeps its copy of the array

// device address of the current device's array; looked up on the first call on that device
int scratch_for_current_device(unsigned char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return ET_EHIP;
  std::lock_guard<std::mutex> hold(g_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ET_EHIP;
    g_scratch_ptr[dev] = (unsigned char*)p;
  }
  *out = g_scratch_ptr[dev];
  return ET_OK;
}

// up to 64 tensors per launch travel as kernel arguments
constexpr int BATCH = 64;
struct TableBatch {
  const float* g[BATCH];
  const unsigned char* w[BATCH];
  const unsigned char* ws[BATCH];
  uint32_t numel[BATCH];
  uint32_t begin[BATCH + 1];   // first chunk of each tensor of the batch, and one past the last
  uint32_t first_tensor, count, wsize;
};

// one workgroup per tensor of the batch writes that tensor's chunks and its offset
__global__ __launch_bounds__(64) void build_table_kernel(TableBatch b, TensorSeg* __restrict__ segs,
                                                         uint32_t* __restrict__ seg_begin) {
  const uint32_t k = blockIdx.x;
  if (k >= b.count) return;
  const uint32_t first = b.begin[k], n_chunks = b.begin[k + 1] - first;
  for (uint32_t ch = threadIdx.x; ch < n_chunks; ch += 64) {
    const size_t off = (size_t)ch * SEG_ELEMS;
    TensorSeg t;
    t.g = b.g[k] + off;
    t.w = b.w[k] + off * b.wsize;
    t.w_snap = b.ws[k] + off * b.wsize;
    t.n = (uint32_t)min((size_t)SEG_ELEMS, (size_t)b.numel[k] - off);
    t.tensor = b.first_tensor + k;
    segs[first + ch] = t;
  }
  if (threadIdx.x == 0) {
    seg_begin[b.first_tensor + k] = first;
    if (k + 1 == b.count) seg_begin[b.first_tensor + k + 1] = b.begin[k + 1];
  }
}

}  // namespace

extern "C" int et_importance_reduce_static(int32_t n, void* const* grad_dev, void* const* w_dev,
                                           void* const* w_snapshot_dev, const uint64_t* numel, int32_t dtype,
                                           void* hip_stream, double* importance_dev) {
  if (n <= 0 || !grad_dev || !w_dev || !w_snapshot_dev || !numel || !importance_dev) return ET_EINVAL;
  if (dtype != ET_F32 && dtype != ET_BF16) return ET_EINVAL;
  if ((uint32_t)n > MAX_STATIC_TENSORS) return ET_ENOMEM;
  if (reinterpret_cast<uintptr_t>(importance_dev) & 7) return ET_EINVAL;
  uint64_t total_segs = 0;
  for (int32_t i = 0; i < n; i++) {
    if (!grad_dev[i] || !w_dev[i] || !w_snapshot_dev[i] || numel[i] == 0 || numel[i] > 0xffffffffull) return ET_EINVAL;
    if ((reinterpret_cast<uintptr_t>(grad_dev[i]) & 3) || (reinterpret_cast<uintptr_t>(w_dev[i]) & 1) ||
        (reinterpret_cast<uintptr_t>(w_snapshot_dev[i]) & 1) ||
        (dtype == ET_F32 && ((reinterpret_cast<uintptr_t>(w_dev[i]) | reinterpret_cast<uintptr_t>(w_snapshot_dev[i])) & 3)))
      return ET_EINVAL;
    total_segs += (numel[i] + SEG_ELEMS - 1) / SEG_ELEMS;
  }
  if (total_segs > MAX_STATIC_SEGS) return ET_ENOMEM;   // beyond the fixed table: use et_importance with a workspace
  unsigned char* base = nullptr;
  const int rc = scratch_for_current_device(&base);
  if (rc != ET_OK) return rc;
  TensorSeg* segs = (TensorSeg*)(base + OFF_SEGS);
  double* partial = (double*)(base + OFF_PARTIAL);
  uint32_t* seg_begin = (uint32_t*)(base + OFF_BEGIN);
  hipStream_t s = (hipStream_t)hip_stream;

  uint32_t next_seg = 0;
  for (int32_t i0 = 0; i0 < n; i0 += BATCH) {
    TableBatch b;
    b.first_tensor = (uint32_t)i0;
    b.count = (uint32_t)std::min<int32_t>(BATCH, n - i0);
    b.wsize = dtype == ET_BF16 ? 2u : 4u;
    for (uint32_t k = 0; k < (uint32_t)BATCH; k++) {
      const bool live = k < b.count;
      b.g[k] = live ? (const float*)grad_dev[i0 + k] : nullptr;
      b.w[k] = live ? (const unsigned char*)w_dev[i0 + k] : nullptr;
      b.ws[k] = live ? (const unsigned char*)w_snapshot_dev[i0 + k] : nullptr;
      b.numel[k] = live ? (uint32_t)numel[i0 + k] : 0u;
      b.begin[k] = next_seg;
      if (live) next_seg += (uint32_t)((numel[i0 + k] + SEG_ELEMS - 1) / SEG_ELEMS);
    }
    b.begin[BATCH] = next_seg;
    // (entries past count repeat the end offset, so begin[count] is the end of the batch's last tensor)
    hipLaunchKernelGGL(build_table_kernel, dim3(b.count), dim3(64), 0, s, b, segs, seg_begin);
    if (hipGetLastError() != hipSuccess) return ET_EHIP;
  }
  if (et::importance_reduce(segs, (int)total_segs, seg_begin, n, dtype == ET_BF16, partial, importance_dev, s, 0) != hipSuccess)
    return ET_EHIP;
  return ET_OK;
}
