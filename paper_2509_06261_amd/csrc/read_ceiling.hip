// Read ceiling of the decode kernel's work decomposition on one GPU (measurement aid, no part of the library).
//
// The MFMA decode kernel is a persistent grid of independent waves (two workgroups of four per compute unit),
// each streaming 8 KiB tiles of K/V out of head chunks scattered over the slab pool, with 16 KiB in flight.
// This program runs kernels that do the same and NOTHING else -- they load and fold the words into one register --
// to tell which part of the distance to the HBM peak belongs to that decomposition rather than to the kernel:
//   pattern   "K operand": per load instruction 16 rows x 64 B, rows 256 B apart (the MFMA A-operand layout of
//             an FP16 K tile); "contiguous": 1 KiB per instruction; "LDS": contiguous 16-byte loads straight to
//             LDS (global_load_lds_dwordx4), read back in the K-operand layout (xor-swizzled, conflict-free)
//   ring      tiles in flight per wave: 2 (16 KiB, the decode kernel's) or 4
//   placement every wave streams its own 32 KiB chunks, which are scattered over the pool in groups of `group`
//             neighbours (1: every chunk elsewhere; 64: 2 MiB pieces); or all waves sweep the pool together
//             (tile t of wave w is tile t * n_waves + w of the pool)
// Build (build.py does it): hipcc --offload-arch=gfx950 -O3 -std=c++17 read_ceiling.hip -o read_ceiling
// Run:   read_ceiling [pool GiB = 32] [32 KiB chunks per wave = 192] [workgroups = 512] [group = 1]
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <utility>
#include <vector>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define RC_GLOBAL __attribute__((address_space(1)))
#define RC_LDS __attribute__((address_space(3)))

namespace {

constexpr int kChunk = 32768, kTile = 8192, kTilesPerChunk = kChunk / kTile, kWaves = 4;
enum { kOperand = 0, kContiguous = 1 };

__device__ __forceinline__ uint32_t fold(u32x4 v) { return v[0] ^ v[1] ^ v[2] ^ v[3]; }

// byte offset, inside an 8 KiB tile, of the 16 bytes lane `lane` loads with instruction i (0..7)
template <int PATTERN>
__device__ __forceinline__ uint32_t lane_offset(int i, int lane) {
  if (PATTERN == kContiguous) return i * 1024 + lane * 16;
  const int j = lane >> 4, c = lane & 15, u = i >> 2, s = i & 3;  // row c of half-tile u, k-step s, 16-byte piece j
  const int row = 8 * (c >> 2) + 4 * u + (c & 3);
  return row * 256 + 16 * j + 64 * s;
}

struct Args {
  const uint8_t* pool;
  const uint32_t* chunk_slot;  // [n_chunks] 32 KiB slot of every chunk, wave-major
  int n_chunks, chunks_per_wave;
  uint32_t* sink;
};

// tile t of this wave (past the end: the last tile again, as the decode kernel's surplus refills)
template <bool TOGETHER>
__device__ __forceinline__ const RC_GLOBAL uint8_t* tile_of(const Args& a, int wave, int n_waves, int t) {
  const int n_tiles = a.chunks_per_wave * kTilesPerChunk;
  const int tt = t < n_tiles ? t : n_tiles - 1;
  if (TOGETHER) return (const RC_GLOBAL uint8_t*)(a.pool + ((size_t)tt * n_waves + wave) * kTile);
  int ch = wave * a.chunks_per_wave + tt / kTilesPerChunk;
  ch = ch < a.n_chunks ? ch : a.n_chunks - 1;
  return (const RC_GLOBAL uint8_t*)(a.pool + (size_t)a.chunk_slot[ch] * kChunk + (size_t)(tt % kTilesPerChunk) * kTile);
}

// one 16-byte load; NT: with the non-temporal hint (read-once data that should not displace anything in the caches)
template <bool NT>
__device__ __forceinline__ u32x4 load16(const RC_GLOBAL uint8_t* p) {
  if (NT) return __builtin_nontemporal_load((const RC_GLOBAL u32x4*)p);
  return *(const RC_GLOBAL u32x4*)p;
}

template <int PATTERN, int RING, bool TOGETHER, bool NT = false>
__global__ __launch_bounds__(256, 2) void read_to_registers(Args a) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n_waves = gridDim.x * kWaves, n_tiles = a.chunks_per_wave * kTilesPerChunk;
  uint32_t acc = 0;
  u32x4 ring[RING][8];
#pragma unroll
  for (int b = 0; b < RING; ++b) {
    const RC_GLOBAL uint8_t* p = tile_of<TOGETHER>(a, wave, n_waves, b);
#pragma unroll
    for (int i = 0; i < 8; ++i) ring[b][i] = load16<NT>(p + lane_offset<PATTERN>(i, lane));
  }
  for (int t = 0; t < n_tiles; t += RING) {
#pragma unroll
    for (int b = 0; b < RING; ++b) {
      __builtin_amdgcn_sched_barrier(0);  // consume a tile, then refill its slot: the order the ring means
#pragma unroll
      for (int i = 0; i < 8; ++i) acc ^= fold(ring[b][i]);
      __builtin_amdgcn_sched_barrier(0);
      const RC_GLOBAL uint8_t* p = tile_of<TOGETHER>(a, wave, n_waves, t + b + RING);
#pragma unroll
      for (int i = 0; i < 8; ++i) ring[b][i] = load16<NT>(p + lane_offset<PATTERN>(i, lane));
    }
  }
  if (acc == 0x12345678u) a.sink[wave] = acc;  // (keeps the loads alive)
}

// The plain way to read a buffer: short-lived workgroups, workgroup g reads the contiguous piece g of PIECE bytes,
// every lane 16 bytes per instruction, all of the piece's loads issued before the first is used.  No tiles, no
// chunks, no persistent waves: what the memory system gives a kernel that does nothing but stream sequentially.
template <int PIECE, bool NT>
__global__ __launch_bounds__(256) void read_sequential(const uint8_t* pool, uint32_t* sink) {
  constexpr int kLoads = PIECE / (256 * 16);
  const RC_GLOBAL uint8_t* p = (const RC_GLOBAL uint8_t*)(pool + (size_t)blockIdx.x * PIECE) + threadIdx.x * 16;
  u32x4 v[kLoads];
#pragma unroll
  for (int i = 0; i < kLoads; ++i) v[i] = load16<NT>(p + i * 4096);
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < kLoads; ++i) acc ^= fold(v[i]);
  if (acc == 0x12345678u) sink[blockIdx.x & 1023] = acc;
}

// 16 distinct values over the 16 rows that one K-operand read touches: the xor swizzle of the LDS columns
__device__ __forceinline__ int swizzle(int row) { return (row & 3) | ((row >> 3) << 2); }

// Ring of two tiles per wave in LDS.  Load instruction i, lane l fills LDS slot 64 i + l = row 4 i + l / 16,
// position l % 16, with the row's 16-byte column (l % 16) ^ swizzle(row): still 256 contiguous bytes per 16 lanes.
__global__ __launch_bounds__(256, 2) void read_through_lds(Args a) {
  extern __shared__ uint8_t smem[];
  const int lane = threadIdx.x & 63;
  const int lw = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wave = blockIdx.x * kWaves + lw;
  const int n_waves = gridDim.x * kWaves, n_tiles = a.chunks_per_wave * kTilesPerChunk;
  uint8_t* mine = smem + lw * 2 * kTile;
  uint32_t acc = 0;
  auto issue = [&](int b, const RC_GLOBAL uint8_t* p) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = 4 * i + (lane >> 4);
      const int col = (lane & 15) ^ swizzle(row);
      __builtin_amdgcn_global_load_lds((const RC_GLOBAL void*)(p + row * 256 + col * 16), (RC_LDS void*)(mine + b * kTile + i * 1024),
                                       16, 0, 0);
    }
  };
  auto consume = [&](int b) {
    const int j = lane >> 4, c = lane & 15;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int u = i >> 2, s = i & 3;
      const int row = 8 * (c >> 2) + 4 * u + (c & 3), col = 4 * s + j;
      acc ^= fold(*(const u32x4*)(mine + b * kTile + row * 256 + ((col ^ swizzle(row)) * 16)));
    }
  };
  issue(0, tile_of<false>(a, wave, n_waves, 0));
  issue(1, tile_of<false>(a, wave, n_waves, 1));
  for (int t = 0; t < n_tiles; t += 2) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");  // the older tile has landed; the younger one's 8 loads may be out
      consume(b);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // read before the slot is refilled
      issue(b, tile_of<false>(a, wave, n_waves, t + b + 2));
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (acc == 0x12345678u) a.sink[wave] = acc;
}

#define RC_CHECK(x)                                                                  \
  do {                                                                               \
    hipError_t e_ = (x);                                                             \
    if (e_ != hipSuccess) {                                                          \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
      return 1;                                                                      \
    }                                                                                \
  } while (0)

}  // namespace

int main(int argc, char** argv) {
  const size_t pool_bytes = (size_t)(argc > 1 ? std::atoi(argv[1]) : 32) << 30;
  const int chunks_per_wave = argc > 2 ? std::atoi(argv[2]) : 192;
  const int n_wg = argc > 3 ? std::atoi(argv[3]) : 512;
  const size_t group = argc > 4 ? (size_t)std::atoi(argv[4]) : 1;
  const int n_waves = n_wg * kWaves;
  const size_t n_chunks = (size_t)n_waves * chunks_per_wave, slots = pool_bytes / kChunk;
  if (chunks_per_wave < 1 || n_wg < 1 || group < 1 || n_chunks > slots || n_chunks > 0x7fffffffu) {
    std::printf("the chunks (%zu) must fit the pool (%zu slots of 32 KiB)\n", n_chunks, slots);
    return 1;
  }
  uint8_t* pool = nullptr;
  uint32_t *chunk_slot = nullptr, *sink = nullptr;
  RC_CHECK(hipMalloc(&pool, pool_bytes));
  RC_CHECK(hipMemset(pool, 1, pool_bytes));
  // groups of `group` neighbouring slots stay together, the groups are shuffled (seeded)
  const size_t n_groups = slots / group;
  std::vector<uint32_t> order(n_groups);
  for (size_t i = 0; i < n_groups; ++i) order[i] = (uint32_t)i;
  uint64_t state = 0x9E3779B97F4A7C15ull;
  for (size_t i = n_groups - 1; i > 0; --i) {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    std::swap(order[i], order[(state >> 33) % (i + 1)]);
  }
  std::vector<uint32_t> slot(n_chunks);
  for (size_t i = 0; i < n_chunks; ++i) slot[i] = (uint32_t)(order[i / group] * group + i % group);
  RC_CHECK(hipMalloc(&chunk_slot, n_chunks * 4));
  RC_CHECK(hipMemcpy(chunk_slot, slot.data(), n_chunks * 4, hipMemcpyHostToDevice));
  RC_CHECK(hipMalloc(&sink, (size_t)(n_waves > 1024 ? n_waves : 1024) * 4));
  hipEvent_t e0, e1;
  RC_CHECK(hipEventCreate(&e0));
  RC_CHECK(hipEventCreate(&e1));
  const size_t lds = (size_t)kWaves * 2 * kTile;
  RC_CHECK(hipFuncSetAttribute((const void*)read_through_lds, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const Args a{pool, chunk_slot, (int)n_chunks, chunks_per_wave, sink};
  const double bytes = (double)n_chunks * kChunk;
  const char* names[] = {"K operand, ring 2", "contiguous, ring 2", "contiguous to LDS, ring 2", "contiguous, ring 4",
                         "K operand, ring 4", "contiguous, ring 2, all waves sweep together",
                         "K operand, ring 2, all waves sweep together", "K operand, ring 2, non-temporal loads",
                         "K operand, ring 4, non-temporal loads", "contiguous, ring 2, non-temporal loads",
                         "contiguous, ring 4, non-temporal loads", "contiguous, ring 2, sweep together, non-temporal",
                         "sequential, 16 KiB per short-lived workgroup", "sequential, 64 KiB per short-lived workgroup",
                         "sequential, 16 KiB, non-temporal loads", "sequential, 32 KiB, non-temporal loads",
                         "sequential, 64 KiB, non-temporal loads", "sequential, 128 KiB, non-temporal loads"};
  constexpr int kModes = 18;
  const auto seq_grid = [&](int piece) { return dim3((unsigned)(bytes / piece)); };  // the same bytes, front of the pool
  for (int mode = 0; mode < kModes; ++mode) {
    float best = 1e30f;
    for (int rep = 0; rep < 4; ++rep) {
      RC_CHECK(hipEventRecord(e0));
      switch (mode) {
        case 0: hipLaunchKernelGGL((read_to_registers<kOperand, 2, false>), dim3(n_wg), dim3(256), 0, 0, a); break;
        case 1: hipLaunchKernelGGL((read_to_registers<kContiguous, 2, false>), dim3(n_wg), dim3(256), 0, 0, a); break;
        case 2: hipLaunchKernelGGL(read_through_lds, dim3(n_wg), dim3(256), lds, 0, a); break;
        case 3: hipLaunchKernelGGL((read_to_registers<kContiguous, 4, false>), dim3(n_wg), dim3(256), 0, 0, a); break;
        case 4: hipLaunchKernelGGL((read_to_registers<kOperand, 4, false>), dim3(n_wg), dim3(256), 0, 0, a); break;
        case 5: hipLaunchKernelGGL((read_to_registers<kContiguous, 2, true>), dim3(n_wg), dim3(256), 0, 0, a); break;
        case 6: hipLaunchKernelGGL((read_to_registers<kOperand, 2, true>), dim3(n_wg), dim3(256), 0, 0, a); break;
        case 7: hipLaunchKernelGGL((read_to_registers<kOperand, 2, false, true>), dim3(n_wg), dim3(256), 0, 0, a); break;
        case 8: hipLaunchKernelGGL((read_to_registers<kOperand, 4, false, true>), dim3(n_wg), dim3(256), 0, 0, a); break;
        case 9: hipLaunchKernelGGL((read_to_registers<kContiguous, 2, false, true>), dim3(n_wg), dim3(256), 0, 0, a); break;
        case 10: hipLaunchKernelGGL((read_to_registers<kContiguous, 4, false, true>), dim3(n_wg), dim3(256), 0, 0, a); break;
        case 11: hipLaunchKernelGGL((read_to_registers<kContiguous, 2, true, true>), dim3(n_wg), dim3(256), 0, 0, a); break;
        case 12: hipLaunchKernelGGL((read_sequential<16384, false>), seq_grid(16384), dim3(256), 0, 0, pool, sink); break;
        case 13: hipLaunchKernelGGL((read_sequential<65536, false>), seq_grid(65536), dim3(256), 0, 0, pool, sink); break;
        case 14: hipLaunchKernelGGL((read_sequential<16384, true>), seq_grid(16384), dim3(256), 0, 0, pool, sink); break;
        case 15: hipLaunchKernelGGL((read_sequential<32768, true>), seq_grid(32768), dim3(256), 0, 0, pool, sink); break;
        case 16: hipLaunchKernelGGL((read_sequential<65536, true>), seq_grid(65536), dim3(256), 0, 0, pool, sink); break;
        default: hipLaunchKernelGGL((read_sequential<131072, true>), seq_grid(131072), dim3(256), 0, 0, pool, sink); break;
      }
      RC_CHECK(hipGetLastError());
      RC_CHECK(hipEventRecord(e1));
      RC_CHECK(hipEventSynchronize(e1));
      float ms = 0.f;
      RC_CHECK(hipEventElapsedTime(&ms, e0, e1));
      if (rep && ms < best) best = ms;  // (the first launch warms up)
    }
    std::printf("%-48s %7.3f ms  %5.2f TB/s\n", names[mode], best, bytes / best / 1e9);
    std::fflush(stdout);
  }
  RC_CHECK(hipFree(pool));
  RC_CHECK(hipFree(chunk_slot));
  RC_CHECK(hipFree(sink));
  return 0;
}
