// What an LDS atomic per logit costs on this GPU, by address pattern: a stand-alone probe of the
// operation that bounds the streaming loop of k_logits_hist (one ds_add_u32 per bf16 logit into a
// 4096-word histogram).  Workgroups of 512 threads, 1 or 4 per CU, issue nothing but atomics (eight
// per lane and iteration, like one 16-byte chunk) on addresses of a given pattern; the result is the
// CU's cycles per wavefront instruction and what that rate would mean in GB/s of bf16 logits per CU.
// Every address is masked to the 16 KB array.  Build and run: python -m paper_2502_13652_amd.lds_atomic_probe
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

constexpr int WORDS = 4096;
enum Pattern { LANE_LINEAR = 0, UNIFORM, HOT_256, RANDOM_ROW_OWN_BANK, WRITE_UNIFORM, READ_UNIFORM, ADD_RTN_UNIFORM, HALF_WAVE_UNIFORM, ADD_U64_UNIFORM, N_PATTERNS };
static const char* const NAMES[N_PATTERNS] = {
    "ds_add_u32, lane-linear (no conflict)", "ds_add_u32, uniform over 4096 words", "ds_add_u32, uniform over 256 words",
    "ds_add_u32, random row, bank = lane mod 32", "ds_write_b32, uniform over 4096 words", "ds_read_b32, uniform over 4096 words",
    "ds_add_rtn_u32, uniform over 4096 words", "ds_add_u32, uniform, 32 of 64 lanes", "ds_add_u64, uniform over 2048 words"};

__device__ __forceinline__ uint32_t mix(uint32_t x) { x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16; return x; }

template <int P>
__global__ __launch_bounds__(512, 8) void k_probe(int iters, uint32_t* out) {
  __shared__ uint32_t h[WORDS + 2];
  for (int i = threadIdx.x; i < WORDS; i += 512) h[i] = 0;
  __syncthreads();
  const uint32_t lane = threadIdx.x & 63, t = threadIdx.x + blockIdx.x * 512;
  uint32_t a[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t r = mix(t * 8 + j + 12345u);
    if (P == LANE_LINEAR) a[j] = (lane + j * 64) & (WORDS - 1);
    else if (P == HOT_256) a[j] = r & 255;
    else if (P == RANDOM_ROW_OWN_BANK) a[j] = ((r & 127) << 5 | (lane & 31)) & (WORDS - 1);
    else if (P == ADD_U64_UNIFORM) a[j] = (r & (WORDS / 2 - 1)) * 2;
    else a[j] = r & (WORDS - 1);
  }
  uint32_t acc = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t ad = a[j];
      if (P == WRITE_UNIFORM) h[ad] = it;
      else if (P == READ_UNIFORM) acc += h[ad];
      else if (P == ADD_RTN_UNIFORM) acc += atomicAdd(&h[ad], 1u);
      else if (P == HALF_WAVE_UNIFORM) { if (lane < 32) atomicAdd(&h[ad], 1u); }
      else if (P == ADD_U64_UNIFORM) atomicAdd((unsigned long long*)&h[ad], 1ull);
      else atomicAdd(&h[ad], 1u);
      // next address of the same pattern
      if (P == LANE_LINEAR || P == RANDOM_ROW_OWN_BANK) a[j] = (ad + 64 * 37) & (WORDS - 1);
      else if (P == HOT_256) a[j] = (ad * 5 + 1 + j) & 255;
      else if (P == ADD_U64_UNIFORM) a[j] = (((ad >> 1) * 5 + 1 + j) * 2) & (WORDS - 1);
      else a[j] = (ad * 5 + 1 + j) & (WORDS - 1);
    }
  }
  __syncthreads();
  if (threadIdx.x < 64) acc += h[threadIdx.x];
  if (acc == 0x12345678u) out[0] = acc;                     // keeps the reads alive
}

template <int P>
int run(int grid, int iters, uint32_t* out, float* ms) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  hipLaunchKernelGGL(k_probe<P>, dim3(grid), dim3(512), 0, 0, iters, out);        // warm-up
  CK(hipEventRecord(e0));
  hipLaunchKernelGGL(k_probe<P>, dim3(grid), dim3(512), 0, 0, iters, out);
  CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  CK(hipEventElapsedTime(ms, e0, e1));
  CK(hipEventDestroy(e0)); CK(hipEventDestroy(e1));
  return 0;
}

int main() {
  uint32_t* out;
  CK(hipMalloc(&out, 64));
  int cus = 0, khz = 0;
  CK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
  CK(hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, 0));
  std::printf("compute units %d, clock %d kHz (cycles below assume it)\n", cus, khz);
  const int iters = 2000;
  for (int per_cu = 4; per_cu >= 1; per_cu -= 3) {
    float ms[N_PATTERNS];
    const int grid = cus * per_cu;
    if (run<LANE_LINEAR>(grid, iters, out, &ms[0]) || run<UNIFORM>(grid, iters, out, &ms[1]) || run<HOT_256>(grid, iters, out, &ms[2]) ||
        run<RANDOM_ROW_OWN_BANK>(grid, iters, out, &ms[3]) || run<WRITE_UNIFORM>(grid, iters, out, &ms[4]) ||
        run<READ_UNIFORM>(grid, iters, out, &ms[5]) || run<ADD_RTN_UNIFORM>(grid, iters, out, &ms[6]) ||
        run<HALF_WAVE_UNIFORM>(grid, iters, out, &ms[7]) || run<ADD_U64_UNIFORM>(grid, iters, out, &ms[8]))
      return 1;
    for (int p = 0; p < N_PATTERNS; ++p) {
      const double instr_per_cu = (double)per_cu * 8 /*waves*/ * iters * 8;
      const double cyc = ms[p] * 1e-3 * (double)khz * 1e3 / instr_per_cu;
      std::printf("%d workgroup(s)/CU  %-44s %7.3f ms  %6.2f cycles per wave instruction and CU  = %5.1f GB/s of bf16 logits per CU\n",
                  per_cu, NAMES[p], ms[p], cyc, instr_per_cu * 128 / (ms[p] * 1e-3) / 1e9);
    }
  }
  CK(hipFree(out));
  return 0;
}
