// Internal declarations shared by the library's translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "tim.h"

#define TIM_D 128          // head dim
#define TIM_PS 16          // tokens per page in the default layout; page size 1 (the paper's) is the other one
#define TIM_G 4            // query heads per KV head
#define TIM_ROW_BYTES 256  // one bf16 row of TIM_D
#define TIM_TILE_BYTES (TIM_PS * TIM_ROW_BYTES)  // one (page, kv head) tile: 4 KiB

struct tim_ctx {
  tim_config cfg;
  tim_state st;
  bool bound;
  int n_cu;
  int attn_impl;  // tim_attn_impl: matrix-core attention (default) or vector-ALU attention
  int attn_cpb;   // target chunks per attention block
  int attn_fill;  // shrink blocks until there are this many per CU
  int block_waves = 0;  // tim_tuning.block_waves: 0 = chosen per launch, else 4, 6, 8 or 12
  int short_per = 0;    // tim_tuning.short_list_chunks: 0 = chosen by the schedule, else chunks per block of a list that is not graded
  double inv_freq[TIM_D / 2];  // theta_i in fp64, computed once on the host
  bool sched_valid = false;    // tim_attn_schedule ran and no call has changed a length since
  int sched_cpb = 0, sched_slots = 0, sched_waves = 4;
  int grade_big = 32, grade_small = 8;  // graded block sizes along the schedule, in 1/16 rounds of work to go
  int round_items = 0;         // tim_tuning.round_items: > 0 = a round of the schedule is this many blocks, and even
                               // launches that fit the chip at once are scheduled (small shapes in tests)
  bool timing_on = false;      // kernel timing for benchmarks (tim_timing_begin / _end)
  int timing_n = 0;
  std::vector<hipEvent_t> ev_start, ev_stop;
};

#define TIM_HIP_CHECK(expr)                  \
  do {                                       \
    hipError_t _e = (expr);                  \
    if (_e != hipSuccess) return TIM_ERR_HIP; \
  } while (0)

#define TIM_LAUNCH_CHECK() TIM_HIP_CHECK(hipGetLastError())

// attn.hip: looks up, for the current device, the address of the array tim_decode_attn_noalloc uses
void tim_noalloc_scratch_init();

static inline hipStream_t tim_hs(tim_stream s) { return reinterpret_cast<hipStream_t>(s); }

// The kernels move K/V rows, queries and outputs in 16-byte pieces and index int32 arrays as such; a
// pointer that is not aligned for that is refused on the host, never handed to a kernel.
static inline bool tim_aligned(const void *p, uintptr_t bytes) { return (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) == 0; }
static inline bool tim_rows_ok(const void *p) { return p != nullptr && tim_aligned(p, 16); }
static inline bool tim_ints_ok(const void *p) { return p != nullptr && tim_aligned(p, 4); }

// words per sequence of the visibility mask: one bit per logical token
__host__ __device__ __forceinline__ int tim_mask_words(const tim_config &cfg) {
  return (cfg.max_pages_per_seq * cfg.page_size + 31) / 32;
}

// K/V tiles are streamed: read (or written) once per call.  Non-temporal accesses do not claim cache
// space for them; on this chip a pure read stream sustains 7.0 TB/s with them against 6.25 TB/s with
// ordinary loads (measured).
typedef unsigned int tim_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 tim_load_stream(const uint4 *p) {
  return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const tim_u32x4 *>(p)));
}
__device__ __forceinline__ void tim_store_stream(uint4 *p, const uint4 &v) {
  __builtin_nontemporal_store(__builtin_bit_cast(tim_u32x4, v), reinterpret_cast<tim_u32x4 *>(p));
}

__device__ __forceinline__ void tim_set_status(int32_t *status, int32_t err) { atomicCAS(status, 0, err); }

// ---- wave / block scans (wave64) -------------------------------------------------
__device__ __forceinline__ int tim_wave_incl_scan(int v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    int o = __shfl_up(v, d, 64);
    if (lane >= d) v += o;
  }
  return v;
}

// Inclusive block scan of one int per thread; blockDim.x <= 1024, multiple of 64.
// `smem` holds at least 17 ints.  Returns the inclusive prefix; *total = block sum.
__device__ __forceinline__ int tim_block_incl_scan(int v, int *smem, int *total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  int incl = tim_wave_incl_scan(v);
  __syncthreads();  // protect smem reuse across calls
  if (lane == 63) smem[w] = incl;
  __syncthreads();
  if (w == 0) {
    int t = lane < nw ? smem[lane] : 0;
    int ti = tim_wave_incl_scan(t);
    if (lane < nw) smem[lane] = ti - t;  // exclusive wave offsets
    if (lane == nw - 1) smem[16] = ti;
  }
  __syncthreads();
  incl += smem[w];
  *total = smem[16];
  return incl;
}
