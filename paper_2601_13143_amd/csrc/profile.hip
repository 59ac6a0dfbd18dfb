// Optional per-kernel timing for benchmarks: HIP events recorded on the launch stream right before and
// after the launches of the selected kinds, accumulated per kind together with the algorithmic work
// (flops or bytes) of each launch.  Off by default; when off a ProfScope costs one load and a branch.
#include <mutex>
#include <vector>

#include "common.hpp"

namespace fastav {

namespace {
struct Rec { hipEvent_t a, b; int kind; double work; };
struct State {
  std::mutex mu;
  uint32_t mask = 0;
  std::vector<hipEvent_t> pool;
  std::vector<Rec> pending;
  double ms[FASTAV_PROF_KIND_COUNT] = {};
  double work[FASTAV_PROF_KIND_COUNT] = {};
  int64_t n[FASTAV_PROF_KIND_COUNT] = {};
};
State g_prof;

hipEvent_t get_event(State& st) {
  if (!st.pool.empty()) { hipEvent_t e = st.pool.back(); st.pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

ProfScope::ProfScope(int kind, double work, hipStream_t s) : rec_(nullptr), stream_(s) {
  if (!(g_prof.mask & (1u << kind))) return;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  hipEvent_t a = get_event(g_prof), b = get_event(g_prof);
  if (!a || !b) return;
  g_prof.pending.push_back(Rec{a, b, kind, work});
  rec_ = (void*)b;                                         // the end event itself: a collect in between may reorder `pending`
  (void)hipEventRecord(a, s);
}

ProfScope::~ProfScope() {
  if (!rec_) return;
  (void)hipEventRecord((hipEvent_t)rec_, stream_);
}

// ---- "achievable peak" probes: what this chip sustains with nothing in the way, next to the datasheet figures.
// A loop of independent bf16 matrix instructions only (no memory traffic inside the loop), two waves per SIMD on
// every CU.  The operand registers are filled once: with small integers, or from `operands` (8 A/B pairs of 16 bytes
// per lane, rotated through) - what a matrix instruction costs in power, and with it the clock the chip holds,
// depends on how many operand bits toggle, so operands drawn like a model's activations give a lower, more honest
// ceiling than constants do (2.05 against 2.46 PFLOP/s on this part).
__global__ __launch_bounds__(256, 2) void k_probe_mfma(int iters, const bf16x8_t* __restrict__ operands, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  bf16x8_t a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (operands != nullptr) {
      a[i] = operands[(2 * i) * 256 + threadIdx.x];
      b[i] = operands[(2 * i + 1) * 256 + threadIdx.x];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) { a[i][e] = (bf16_t)(float)((lane + e) & 3); b[i][e] = (bf16_t)(float)((lane * 3 + e) & 1); }
    }
  }
  f32x4_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[(i + u) & 7], acc[i], 0, 0, 0);
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) t += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  if (t == -1.2345e30f) sink[blockIdx.x * 256 + threadIdx.x] = t;      // never true in practice: keeps the loop alive
}

// A plain streaming read: every lane loads 16 bytes per step, workgroups walk memory in launch order.
__global__ __launch_bounds__(256) void k_probe_read(const f32x4_t* __restrict__ src, int64_t n16, float* __restrict__ sink) {
  f32x4_t s = {0.f, 0.f, 0.f, 0.f};
  const int64_t stride = (int64_t)gridDim.x * 256 * 4;
  int64_t i = ((int64_t)blockIdx.x * 4) * 256 + threadIdx.x;
  for (; i + 3 * 256 < n16; i += stride) {
    const f32x4_t v0 = src[i], v1 = src[i + 256], v2 = src[i + 512], v3 = src[i + 768];
    s[0] += v0[0] + v1[1] + v2[2] + v3[3];
    s[1] += v0[1] + v1[2] + v2[3] + v3[0];
    s[2] += v0[2] + v1[3] + v2[0] + v3[1];
    s[3] += v0[3] + v1[0] + v2[1] + v3[2];
  }
  if (s[0] + s[1] + s[2] + s[3] == -1.2345e30f) sink[blockIdx.x] = s[0];
}

}  // namespace fastav

using namespace fastav;

extern "C" {

fastav_status_t fastav_profile_enable(uint32_t kind_mask) {
  if (kind_mask >> FASTAV_PROF_KIND_COUNT) return fail(FASTAV_EINVAL, "profile: unknown kind bit");
  std::lock_guard<std::mutex> lk(g_prof.mu);
  g_prof.mask = kind_mask;
  return FASTAV_OK;
}

static fastav_status_t drain_locked() {
  for (Rec& r : g_prof.pending) {
    hipError_t e = hipEventSynchronize(r.b);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
    if (e != hipSuccess) { g_prof.pending.clear(); return fail(FASTAV_EHIP, "profile: %s", hipGetErrorString(e)); }
    g_prof.ms[r.kind] += ms; g_prof.work[r.kind] += r.work; g_prof.n[r.kind] += 1;
    g_prof.pool.push_back(r.a); g_prof.pool.push_back(r.b);
  }
  g_prof.pending.clear();
  return FASTAV_OK;
}

fastav_status_t fastav_profile_collect(int32_t kind, double* total_ms, int64_t* launches, double* total_work) {
  if (kind < 0 || kind >= FASTAV_PROF_KIND_COUNT) return fail(FASTAV_EINVAL, "profile: bad kind");
  std::lock_guard<std::mutex> lk(g_prof.mu);
  fastav_status_t st = drain_locked();
  if (st != FASTAV_OK) return st;
  if (total_ms) *total_ms = g_prof.ms[kind];
  if (launches) *launches = g_prof.n[kind];
  if (total_work) *total_work = g_prof.work[kind];
  return FASTAV_OK;
}

fastav_status_t fastav_probe_mfma(int32_t iters, const void* operands, float* sink, double* flops_out, void* stream) {
  if (iters < 1 || !sink) return fail(FASTAV_EINVAL, "probe: iters must be >= 1 and sink non-NULL");
  if (operands && ((uintptr_t)operands % 16)) return fail(FASTAV_EINVAL, "probe: operands must be 16-byte aligned");
  const int blocks = 2048;                                      // 8 workgroups of 4 waves per CU
  hipLaunchKernelGGL(k_probe_mfma, dim3(blocks), dim3(256), 0, (hipStream_t)stream, iters, (const bf16x8_t*)operands, sink);
  if (flops_out) *flops_out = (double)blocks * 4.0 * iters * 32.0 * (2.0 * 16 * 16 * 32);
  return check_launch("probe_mfma");
}

fastav_status_t fastav_probe_read(const void* src, size_t bytes, float* sink, void* stream) {
  if (!src || !sink || bytes < 16384 || ((uintptr_t)src % 16)) return fail(FASTAV_EINVAL, "probe: src (16-byte aligned, >= 16 KB) and sink must be given");
  const int64_t n16 = (int64_t)(bytes / 16);
  int64_t blocks = n16 / 1024;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(k_probe_read, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const f32x4_t*)src, n16, sink);
  return check_launch("probe_read");
}

fastav_status_t fastav_profile_reset(void) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  fastav_status_t st = drain_locked();
  for (int i = 0; i < FASTAV_PROF_KIND_COUNT; ++i) { g_prof.ms[i] = 0; g_prof.work[i] = 0; g_prof.n[i] = 0; }
  return st;
}

}  // extern "C"
