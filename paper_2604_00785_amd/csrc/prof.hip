// Library identification, launch error check, the optional per-kernel
// event timing used by benchmarks, and a probe of the matrix-pipe rate the chip
// sustains for given operand values.
#include <string.h>
#include <string>
#include <vector>
#include "common.h"

namespace {
struct Entry {
  std::string name;
  std::vector<hipEvent_t> starts, stops;
};
bool g_on = false;
std::vector<Entry> g_entries;
std::vector<hipEvent_t> g_pool;

hipEvent_t take_event() {
  if (!g_pool.empty()) {
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
void clear_entries() {
  for (auto& en : g_entries) {
    for (auto e : en.starts) g_pool.push_back(e);
    for (auto e : en.stops) g_pool.push_back(e);
  }
  g_entries.clear();
}
}  // namespace

MoeLaunchScope::MoeLaunchScope(const char* name, hipStream_t s) : slot(-1), stream(s) {
  if (!g_on) return;
  int idx = -1;
  for (size_t i = 0; i < g_entries.size(); ++i)
    if (g_entries[i].name == name) { idx = static_cast<int>(i); break; }
  if (idx < 0) {
    g_entries.push_back(Entry{name, {}, {}});
    idx = static_cast<int>(g_entries.size()) - 1;
  }
  hipEvent_t a = take_event(), b = take_event();
  if (!a || !b) return;
  g_entries[idx].starts.push_back(a);
  g_entries[idx].stops.push_back(b);
  slot = idx;
  (void)hipEventRecord(a, stream);
}
MoeLaunchScope::~MoeLaunchScope() {
  if (slot < 0) return;
  (void)hipEventRecord(g_entries[slot].stops.back(), stream);
}

int moe_check_launch() { return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH; }

namespace {
// Nothing but v_mfma_f32_16x16x32_bf16, the form the grouped GEMM uses: every lane keeps 4 + 2 operand fragments
// in registers (8 accumulators of 16x16) and multiplies them over and over.  No memory traffic inside the loop,
// so the rate measured is the matrix pipe's at the clock the chip holds for these operand values.
__device__ long long g_ceiling_clk[2];
__global__ __launch_bounds__(512) void mfma_ceiling_kernel(const uint16_t* __restrict__ a, const uint16_t* __restrict__ b,
                                                           int iters, float* __restrict__ sink) {
  const size_t t = static_cast<size_t>(blockIdx.x) * 512 + threadIdx.x;
  bf16x8_t fa[4], fb[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) fa[i] = *reinterpret_cast<const bf16x8_t*>(a + t * 32 + i * 8);
#pragma unroll
  for (int j = 0; j < 2; ++j) fb[j] = *reinterpret_cast<const bf16x8_t*>(b + t * 16 + j * 8);
  f32x4_t acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
  const long long w0 = wall_clock64(), c0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
  }
  const long long c1 = __builtin_readcyclecounter(), w1 = wall_clock64();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) s += acc[i][j][r];
  sink[t] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    g_ceiling_clk[0] = c1 - c0;   // core clock cycles
    g_ceiling_clk[1] = w1 - w0;   // 100 MHz ticks
  }
}
// Streaming-read probe: every workgroup reads whole 16 KB blocks of the buffer with 16-byte loads, four in
// flight per lane, and folds them into one word per thread: what the memory system delivers to a kernel that
// does nothing but read.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t blocks, uint32_t* __restrict__ sink) {
  uint32_t acc = 0;
  for (size_t b = blockIdx.x; b < blocks; b += gridDim.x) {
    const uint4* p = src + b * 1024 + threadIdx.x;
    uint4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {   // non-temporal, as the row movers read their rows
      typedef unsigned int u32x4_nt __attribute__((ext_vector_type(4)));
      const u32x4_nt w = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(p + j * 256));
      v[j] = make_uint4(w.x, w.y, w.z, w.w);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
  }
  sink[static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x] = acc;
}
}  // namespace

extern "C" {

const char* moe_version(void) { return "moe_hotpath 0.1 (gfx950, bf16 MFMA)"; }

int moe_prof_enable(int on) {
  clear_entries();
  g_on = on != 0;
  return MOE_OK;
}
int moe_prof_count(void) { return static_cast<int>(g_entries.size()); }

int moe_prof_read(int index, char* name, int name_cap, float* total_ms, int* launches) {
  if (index < 0 || index >= static_cast<int>(g_entries.size()) || !name || name_cap <= 0 || !total_ms || !launches)
    return MOE_ERR_INVALID;
  Entry& en = g_entries[index];
  float total = 0.f;
  for (size_t i = 0; i < en.starts.size(); ++i) {
    if (hipEventSynchronize(en.stops[i]) != hipSuccess) return MOE_ERR_LAUNCH;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, en.starts[i], en.stops[i]) != hipSuccess) return MOE_ERR_LAUNCH;
    total += ms;
  }
  strncpy(name, en.name.c_str(), static_cast<size_t>(name_cap) - 1);
  name[name_cap - 1] = '\0';
  *total_ms = total;
  *launches = static_cast<int>(en.starts.size());
  return MOE_OK;
}

int moe_prof_mfma_ceiling(const moe_bf16* a, const moe_bf16* b, int workgroups, int iters, float* sink,
                          float* ms, double* flop, double* clock_ghz, void* stream) {
  if (!a || !b || !sink || !ms || !flop || !clock_ghz || workgroups <= 0 || iters <= 0) return MOE_ERR_INVALID;
  if (!moe_aligned16(a) || !moe_aligned16(b)) return MOE_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0 = take_event(), e1 = take_event();
  if (!e0 || !e1) return MOE_ERR_LAUNCH;
  (void)hipEventRecord(e0, s);
  hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(workgroups), dim3(512), 0, s, a, b, iters, sink);
  (void)hipEventRecord(e1, s);
  int rc = MOE_OK;
  long long clk[2] = {0, 0};
  if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(ms, e0, e1) != hipSuccess ||
      hipMemcpyFromSymbol(clk, HIP_SYMBOL(g_ceiling_clk), sizeof(clk)) != hipSuccess)
    rc = MOE_ERR_LAUNCH;
  g_pool.push_back(e0);
  g_pool.push_back(e1);
  *flop = 2.0 * 16 * 16 * 32 * 8.0 * iters * 8.0 * workgroups;
  *clock_ghz = clk[1] > 0 ? static_cast<double>(clk[0]) / (static_cast<double>(clk[1]) * 10.0) : 0.0;
  return rc == MOE_OK ? moe_check_launch() : rc;
}

int moe_prof_stream_read(const void* src, size_t bytes, uint32_t* sink, int workgroups, void* stream) {
  if (!src || !sink || workgroups <= 0 || bytes < 16384 || !moe_aligned16(src)) return MOE_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  MOE_LAUNCH("stream_read", stream_read_kernel, dim3(workgroups), dim3(256), 0, s, static_cast<const uint4*>(src),
             bytes / 16384, sink);
  return moe_check_launch();
}

}  // extern "C"
