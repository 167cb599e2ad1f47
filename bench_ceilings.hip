// Secondary ceilings of the histogram build on this part, measured beside the HBM roofline:
//   (1) the rate of local-memory atomics (the scatter-add of Alg. 1's inner loop; App. A.1 / App. B.3
//       discuss its cost on older parts) -- 64-bit / 32-bit integer adds, float adds and the
//       read-and-clear exchange of the drain, conflict-free (the build kernel's slot-rotated address
//       pattern), on random cells and with every lane on ONE cell (the constant-feature worst case of
//       App. A.3), and with a fraction of the lanes switched off (what a skip of a frequent bin or a
//       most-recent-bin register path, App. A.4, would turn the instruction stream into);
//   (2) the rate of a pure streaming read of feature tiles with the build kernel's load shape
//       (16 bytes per lane, 1-KiB runs per wavefront, persistent workgroups, requests one step ahead).
// Stand-alone program (no torch): `bench_ceilings [--mb 800]` prints one table line per measurement.
// Cycle figures use the shader clock measured inside the kernels (cycle counter against the constant
// 100 MHz real-time counter), printed beside them.
#include <hip/hip_runtime.h>

#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#define CK(x)                                                                          \
  do {                                                                                 \
    hipError_t e_ = (x);                                                               \
    if (e_ != hipSuccess) {                                                            \
      printf("HIP error %s at line %d: %s\n", hipGetErrorString(e_), __LINE__, #x);    \
      return 1;                                                                        \
    }                                                                                  \
  } while (0)

namespace {

constexpr int kThreads = 512;
constexpr int kCells = 8192;  // 64 KiB of 64-bit cells: 256 bins x 32 slots, two workgroups per CU
constexpr int kIters = 192;
constexpr int kPerIter = 32;  // atomics per lane and iteration

enum Op { kAddU64 = 0, kAddU32 = 1, kAddF32 = 2, kXchgB64 = 3 };
// kSlotRotated: the build kernel's pattern -- the lanes served together hit different slots, but the
// four rows of a wavefront that share a slot may share a bin (same address inside one instruction);
// kSlotRotatedDistinct: the same with those four rows forced onto different bins (never the same
// address inside one instruction), to see what the same-address cases cost.
enum Pattern { kSlotRotated = 0, kRandomCell = 1, kOneCell = 2, kSlotRotatedDistinct = 3 };

struct Clock {
  unsigned long long cycles, realtime;
};

// active_num / 8 of the lanes take part in each atomic (a fixed set per lane and atomic of the
// iteration); group_mode 1: whole aligned groups of 16 lanes are on or off together.  The loop is
// kept as lean as the build kernel's (one byte-permute per address, two more vector instructions
// for the lane mask when MASKED), so that the local-memory pipe, not the vector units, is what the
// timing sees: a CU issues one vector instruction per SIMD and clock, i.e. the 16 wavefronts of two
// workgroups can afford about 6 vector instructions per atomic before they, and not the 6-7 cycles
// of the atomic, bound the loop.
template <int OP, int PATTERN, bool MASKED>
__global__ void __launch_bounds__(kThreads)
lds_atomic_kernel(const uint32_t* __restrict__ seeds, int active_num, int group_mode, Clock* clk,
                  float* sink) {
  extern __shared__ __align__(16) unsigned long long lds[];
  for (int i = threadIdx.x; i < kCells; i += kThreads) lds[i] = 0ull;
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int j = lane & 3, rho = lane >> 2;
  uint32_t x = seeds[blockIdx.x * kThreads + threadIdx.x];
  // which of the kPerIter atomics of an iteration this lane (or its group of 16) takes part in
  uint32_t mask_bits = 0;
  {
    uint32_t m = seeds[blockIdx.x * kThreads + (group_mode ? (threadIdx.x & ~15) : threadIdx.x)] * 2246822519u;
    for (int k = 0; k < kPerIter; ++k) {
      m = m * 1664525u + 1013904223u;
      if (((m >> 13) & 7u) < (uint32_t)active_num) mask_bits |= 1u << k;
    }
  }
  // byte-permute selectors and the table of 8 * slot, as in the build kernel: in step k a lane of
  // row rho takes byte (rho + k) mod 4 of its word, slot = j + 4 * byte (+ 16 for the second word)
  uint32_t sel[4], tbl[2];
  for (int k = 0; k < 4; ++k) {
    const uint32_t q = (uint32_t)(rho + k) & 3u;
    sel[k] = 0x0c0c0000u | ((4u + q) << 8) | q;
  }
  for (int v = 0; v < 2; ++v) {
    uint32_t t = 0;
    for (int q = 0; q < 4; ++q) t |= (uint32_t)(8 * (16 * v + j + 4 * q)) << (8 * q);
    tbl[v] = t;
  }
  char* cells = reinterpret_cast<char*>(lds);
  const unsigned long long add64 = 0x0000002000000401ull;
  unsigned long long fold = 0;
  unsigned long long c0 = 0, r0 = 0;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    c0 = __builtin_readcyclecounter();
    r0 = wall_clock64();
  }
  for (int it = 0; it < kIters; ++it) {
#pragma unroll
    for (int w = 0; w < kPerIter / 4; ++w) {
      x = x * 1664525u + 1013904223u;
      const uint32_t y = x ^ (x >> 13);  // four random bins
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        uint32_t a;
        if (PATTERN == kSlotRotated) {
          a = __builtin_amdgcn_perm(y, tbl[w & 1], sel[k]);  // (bin << 8) | 8 * slot
        } else if (PATTERN == kSlotRotatedDistinct) {
          a = __builtin_amdgcn_perm(y, tbl[w & 1], sel[k]);
          a = (a & ~0x300u) | ((uint32_t)(rho >> 2) << 8);  // bin mod 4 = row / 4
        } else if (PATTERN == kRandomCell) {
          a = (__builtin_amdgcn_perm(y, y, sel[k]) & 0x1fffu) << 3;  // any of the 8192 cells
        } else {
          a = 8u * 77u;
        }
        const bool on = !MASKED || (mask_bits & (1u << (4 * w + k))) != 0u;
        if (on) {
          if (OP == kAddU64) {
            __hip_atomic_fetch_add(reinterpret_cast<unsigned long long*>(cells + a), add64, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
          } else if (OP == kAddU32) {
            __hip_atomic_fetch_add(reinterpret_cast<unsigned int*>(cells + a), 1025u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
          } else if (OP == kAddF32) {
            __hip_atomic_fetch_add(reinterpret_cast<float*>(cells + a), 1.25f, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
          } else {
            fold += __hip_atomic_exchange(reinterpret_cast<unsigned long long*>(cells + a), 0ull, __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_WORKGROUP);
          }
        }
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clk->cycles = __builtin_readcyclecounter() - c0;
    clk->realtime = wall_clock64() - r0;
  }
  __syncthreads();
  unsigned long long s = fold;
  for (int i = threadIdx.x; i < kCells; i += kThreads) s += lds[i];
  if (s == 12345ull) sink[0] = 1.0f;
}

// Streaming read of n_tiles tiles of n_rows x 64 bytes with the build kernel's load shape: a workgroup
// of 512 threads takes epochs of 512 rows of its tile (its wavefronts 64 rows each, 16 rows = 1 KiB
// per load instruction, 16 bytes per lane), requested one epoch ahead.
__global__ void __launch_bounds__(kThreads)
stream_read_kernel(const uint8_t* __restrict__ base, uint32_t n_rows, int n_tiles, int wgs, uint32_t* sink) {
  const int t = blockIdx.x % n_tiles, p = blockIdx.x / n_tiles;
  const uint8_t* tile = base + (size_t)t * n_rows * 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t n_epochs = n_rows / 512;
  uint32_t acc = 0;
  uint4 w[4], v[4];
  auto load = [&](uint4 (&d)[4], uint32_t e) {
    const uint32_t row0 = e * 512 + wave * 64 + (lane >> 2);
#pragma unroll
    for (int g = 0; g < 4; ++g)
      d[g] = *reinterpret_cast<const uint4*>(tile + (size_t)(row0 + g * 16) * 64 + (lane & 3) * 16);
  };
  uint32_t e = p;
  if (e < n_epochs) load(w, e);
  for (; e < n_epochs; e += wgs) {
    const uint32_t en = e + wgs < n_epochs ? e + wgs : e;
    load(v, en);
#pragma unroll
    for (int g = 0; g < 4; ++g) acc ^= w[g].x ^ w[g].y ^ w[g].z ^ w[g].w;
#pragma unroll
    for (int g = 0; g < 4; ++g) w[g] = v[g];
  }
  if (acc == 0x12345678u) sink[0] = acc;
}

struct Ctx {
  uint32_t* seeds = nullptr;
  Clock* clk = nullptr;
  float* sink = nullptr;
  int cus = 256;
};

template <int OP, int PATTERN, bool MASKED = false>
int run_lds(const Ctx& c, const char* name, int active_num, int group_mode) {
  const size_t lds_bytes = (size_t)kCells * 8;
  int occ = 0;
  CK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, (const void*)lds_atomic_kernel<OP, PATTERN, MASKED>, kThreads,
                                                  lds_bytes));
  if (occ < 1) occ = 1;
  const int blocks = c.cus * occ * 2;  // two rounds of resident workgroups
  hipEvent_t a, b;
  CK(hipEventCreate(&a));
  CK(hipEventCreate(&b));
  for (int rep = 0; rep < 2; ++rep) {  // the first launch warms up
    CK(hipEventRecord(a));
    hipLaunchKernelGGL((lds_atomic_kernel<OP, PATTERN, MASKED>), dim3(blocks), dim3(kThreads), lds_bytes, 0, c.seeds,
                       active_num, group_mode, c.clk, c.sink);
    CK(hipGetLastError());
    CK(hipEventRecord(b));
    CK(hipEventSynchronize(b));
  }
  float ms = 0.0f;
  CK(hipEventElapsedTime(&ms, a, b));
  Clock h;
  CK(hipMemcpy(&h, c.clk, sizeof h, hipMemcpyDeviceToHost));
  const double mhz = h.realtime ? (double)h.cycles / (double)h.realtime * 100.0 : 0.0;
  const double instr = (double)blocks * (kThreads / 64) * kIters * kPerIter;  // wavefront instructions
  const double cyc = ms * 1e-3 * mhz * 1e6 * c.cus / instr;
  const double lanes = 64.0 * active_num / 8.0 / cyc;
  printf("| %-17s | %-18s | %d/8 %-6s | %d | %8.3f | %6.0f | %6.2f | %6.2f |\n", name,
         PATTERN == kSlotRotated ? "slot-rotated"
                                 : (PATTERN == kRandomCell ? "random cell"
                                                           : (PATTERN == kOneCell ? "one cell" : "slot-rot. distinct")),
         active_num,
         group_mode ? "groups" : "lanes", occ, ms, mhz, cyc, lanes);
  fflush(stdout);
  CK(hipEventDestroy(a));
  CK(hipEventDestroy(b));
  return 0;
}

}  // namespace

int main(int argc, char** argv) {
  size_t mb = 800;
  for (int i = 1; i + 1 < argc; ++i)
    if (!strcmp(argv[i], "--mb")) mb = (size_t)atol(argv[i + 1]);
  Ctx c;
  int dev = 0;
  CK(hipGetDevice(&dev));
  CK(hipDeviceGetAttribute(&c.cus, hipDeviceAttributeMultiprocessorCount, dev));
  const int max_blocks = c.cus * 4 * 2;
  std::vector<uint32_t> h((size_t)max_blocks * kThreads);
  for (size_t i = 0; i < h.size(); ++i) {
    uint32_t v = (uint32_t)i * 2654435761u + 12345u;
    v ^= v >> 15;
    v *= 2246822519u;
    v ^= v >> 13;
    h[i] = v;
  }
  CK(hipMalloc(&c.seeds, h.size() * 4));
  CK(hipMalloc(&c.clk, sizeof(Clock)));
  CK(hipMalloc(&c.sink, 16));
  CK(hipMemcpy(c.seeds, h.data(), h.size() * 4, hipMemcpyHostToDevice));
  CK(hipMemset(c.clk, 0, sizeof(Clock)));

  printf("compute units: %d\n", c.cus);
  printf("| instruction | addresses | active | WG/CU | ms | MHz | cycles per wavefront instruction per CU | "
         "active lanes per clock per CU |\n|---|---|---|---|---|---|---|---|\n");
  if (run_lds<kAddU64, kSlotRotated>(c, "ds_add_u64", 8, 0)) return 1;
  if (run_lds<kAddU64, kSlotRotatedDistinct>(c, "ds_add_u64", 8, 0)) return 1;
  if (run_lds<kAddU64, kRandomCell>(c, "ds_add_u64", 8, 0)) return 1;
  if (run_lds<kAddU64, kOneCell>(c, "ds_add_u64", 8, 0)) return 1;
  if (run_lds<kAddU32, kSlotRotated>(c, "ds_add_u32", 8, 0)) return 1;
  if (run_lds<kAddU32, kOneCell>(c, "ds_add_u32", 8, 0)) return 1;
  if (run_lds<kAddF32, kSlotRotated>(c, "ds_add_f32", 8, 0)) return 1;
  if (run_lds<kAddF32, kOneCell>(c, "ds_add_f32", 8, 0)) return 1;
  if (run_lds<kXchgB64, kSlotRotated>(c, "ds_wrxchg_rtn_b64", 8, 0)) return 1;
  for (int act : {8, 6, 4, 3, 2, 1}) {
    if (run_lds<kAddU64, kSlotRotated, true>(c, "ds_add_u64", act, 0)) return 1;
  }
  for (int act : {6, 4, 2}) {
    if (run_lds<kAddU64, kSlotRotated, true>(c, "ds_add_u64", act, 1)) return 1;
  }

  // streaming read
  const int n_tiles = 32;
  uint32_t n_rows = (uint32_t)(mb * 1000000ull / (64ull * n_tiles) / 512 * 512);
  const size_t bytes = (size_t)n_rows * 64 * n_tiles;
  void* buf = nullptr;
  uint32_t* sink = nullptr;
  CK(hipMalloc(&buf, bytes));
  CK(hipMalloc(&sink, 4));
  CK(hipMemset(buf, 1, bytes));
  printf("\nstreaming read of %d tiles x %u rows x 64 B = %.1f MB, 512 threads per workgroup\n", n_tiles, n_rows,
         bytes / 1e6);
  printf("| workgroups per tile | workgroups | ms (median of 9) | GB/s |\n|---|---|---|---|\n");
  hipEvent_t a, b;
  CK(hipEventCreate(&a));
  CK(hipEventCreate(&b));
  for (int wgs : {8, 16, 24, 32, 48, 64}) {
    std::vector<float> t;
    for (int rep = 0; rep < 10; ++rep) {
      CK(hipEventRecord(a));
      hipLaunchKernelGGL(stream_read_kernel, dim3(n_tiles * wgs), dim3(kThreads), 0, 0, (const uint8_t*)buf, n_rows,
                         n_tiles, wgs, sink);
      CK(hipGetLastError());
      CK(hipEventRecord(b));
      CK(hipEventSynchronize(b));
      float ms = 0.0f;
      CK(hipEventElapsedTime(&ms, a, b));
      if (rep) t.push_back(ms);
    }
    for (size_t i = 0; i < t.size(); ++i)
      for (size_t k = i + 1; k < t.size(); ++k)
        if (t[k] < t[i]) {
          const float s = t[i];
          t[i] = t[k];
          t[k] = s;
        }
    const float med = t[t.size() / 2];
    printf("| %d | %d | %.4f | %.0f |\n", wgs, n_tiles * wgs, med, bytes / med / 1e6);
    fflush(stdout);
  }
  return 0;
}
