// Micro-benchmarks of the gfx950 rates the rollout kernels are designed around: how fast one SIMD
// issues bf16 matrix-core and vector-ALU instructions, whether the two overlap inside one wavefront
// or only between wavefronts, what a transcendental, an LDS read and a workgroup barrier cost.
// Not part of the product path: `bench.py --peaks` runs them and prints the figures that the design
// notes quote beside the published peaks.
//
// Every kernel runs `iters` iterations of a fixed straight-line body of inline assembly (so the
// compiler can neither drop nor reorder it) and reports the shader-clock cycles wavefront 0 of
// workgroup 0 spent in the loop.  The bodies touch registers and a static LDS array only; the
// one global store at the end goes to a slot indexed by the thread id.  Results of the arithmetic
// are meaningless on purpose (the required wait states between dependent matrix-core and vector
// instructions are not inserted: nothing reads a value it depends on for an address).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define MFMA_V(acc, a, b) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b))
#define MFMA_A(acc, a, b) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b))
#define MFMA_WA(acc, a, b) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "a"(a), "v"(b))
#define FMA(x, y, z) asm volatile("v_fma_f32 %0, %1, %2, %0" : "+v"(x) : "v"(y), "v"(z))
#define EXP2(x) asm volatile("v_exp_f32 %0, %0" : "+v"(x))
#define RCP(x) asm volatile("v_rcp_f32 %0, %0" : "+v"(x))
#define TANH(v) asm volatile("v_mul_f32 %0, 0x4038aa3b, %0\n v_exp_f32 %0, %0\n v_add_f32 %0, 1.0, %0\n v_rcp_f32 %0, %0\n v_fma_f32 %0, %0, -2.0, 1.0" : "+v"(v))

enum Test : int {
  T_MFMA = 0,          // 16 independent-accumulator MFMAs per iteration (4 accumulators round robin), accumulators in VGPRs
  T_MFMA_AGPR,         // the same with the accumulators in the accumulation-register half
  T_MFMA_WAGPR,        // weights (A operand) read from the accumulation-register half, accumulators in VGPRs: the rollout kernel's form
  T_FMA,               // 32 v_fma_f32 on 8 independent registers
  T_MIX_1_1,           // (1 MFMA, 1 FMA) x 16, all independent: does the vector ALU run under the matrix core in ONE wavefront?
  T_MIX_1_2,           // (1 MFMA, 2 FMA) x 16
  T_MIX_1_4,           // (1 MFMA, 4 FMA) x 16
  T_SPLIT,             // two wavefronts per SIMD: even ones run the T_MFMA body, odd ones 64 FMAs - overlap BETWEEN wavefronts
  T_EXP,               // 32 v_exp_f32 on 8 registers
  T_RCP,               // 32 v_rcp_f32 on 8 registers
  T_MIX_EXP,           // (1 MFMA, 1 v_exp_f32) x 16
  T_TANH,              // 16 x tanh(x) = 1 - 2 / (exp2(2 log2(e) x) + 1): mul, exp, add, rcp, fma
  T_LDS_READ,          // 32 ds_read_b128 (conflict-free, 1 KiB per wavefront each), waited for once per iteration
  T_LDS_CHAIN,         // 8 dependent ds_read_b32 (each address comes from the previous value): LDS latency
  T_BARRIER,           // 8 workgroup barriers
  T_EXCHANGE,          // 4 x (ds_write_b64, barrier, ds_read_b128, wait): one activation hand-over between wavefronts
  T_COUNT
};

__device__ __forceinline__ uint64_t now() { return __builtin_readcyclecounter(); }

template <int TEST>
__global__ __launch_bounds__(512) void bench_kernel(int iters, uint64_t* __restrict__ cycles, float* __restrict__ sink) {
  __shared__ __align__(16) uint32_t lds[16384];        // 64 KiB
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int k = tid; k < 16384; k += blockDim.x) lds[k] = (uint32_t)((k * 4 + 64) & 0xFFFC);   // chain: every word holds an in-bounds byte offset
  __syncthreads();
  f32x4 acc0 = {0, 0, 0, 0}, acc1 = acc0, acc2 = acc0, acc3 = acc0;
  bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u});
  bf16x8 b = a;
  float x0 = 1.0f + lane, x1 = 2.0f, x2 = 3.0f, x3 = 4.0f, x4 = 5.0f, x5 = 6.0f, x6 = 7.0f, x7 = 8.0f;
  const float y = 1.0000001f, z = 1e-9f;
  uint32_t addr = (uint32_t)(lane * 16), chain = (uint32_t)(lane * 4);
  u32x4 r0 = {0, 0, 0, 0}, r1 = r0, r2 = r0, r3 = r0, r4 = r0, r5 = r0, r6 = r0, r7 = r0;
  const uint64_t t0 = now();
  for (int it = 0; it < iters; ++it) {
    if constexpr (TEST == T_MFMA || TEST == T_MFMA_AGPR || TEST == T_MFMA_WAGPR) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if constexpr (TEST == T_MFMA) { MFMA_V(acc0, a, b); MFMA_V(acc1, a, b); MFMA_V(acc2, a, b); MFMA_V(acc3, a, b); }
        if constexpr (TEST == T_MFMA_AGPR) { MFMA_A(acc0, a, b); MFMA_A(acc1, a, b); MFMA_A(acc2, a, b); MFMA_A(acc3, a, b); }
        if constexpr (TEST == T_MFMA_WAGPR) { MFMA_WA(acc0, a, b); MFMA_WA(acc1, a, b); MFMA_WA(acc2, a, b); MFMA_WA(acc3, a, b); }
      }
    } else if constexpr (TEST == T_FMA) {
#pragma unroll
      for (int k = 0; k < 4; ++k) { FMA(x0, y, z); FMA(x1, y, z); FMA(x2, y, z); FMA(x3, y, z); FMA(x4, y, z); FMA(x5, y, z); FMA(x6, y, z); FMA(x7, y, z); }
    } else if constexpr (TEST == T_MIX_1_1) {
#pragma unroll
      for (int k = 0; k < 4; ++k) { MFMA_V(acc0, a, b); FMA(x0, y, z); MFMA_V(acc1, a, b); FMA(x1, y, z); MFMA_V(acc2, a, b); FMA(x2, y, z); MFMA_V(acc3, a, b); FMA(x3, y, z); }
    } else if constexpr (TEST == T_MIX_1_2) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        MFMA_V(acc0, a, b); FMA(x0, y, z); FMA(x4, y, z); MFMA_V(acc1, a, b); FMA(x1, y, z); FMA(x5, y, z);
        MFMA_V(acc2, a, b); FMA(x2, y, z); FMA(x6, y, z); MFMA_V(acc3, a, b); FMA(x3, y, z); FMA(x7, y, z);
      }
    } else if constexpr (TEST == T_MIX_1_4) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        MFMA_V(acc0, a, b); FMA(x0, y, z); FMA(x1, y, z); FMA(x2, y, z); FMA(x3, y, z);
        MFMA_V(acc1, a, b); FMA(x4, y, z); FMA(x5, y, z); FMA(x6, y, z); FMA(x7, y, z);
        MFMA_V(acc2, a, b); FMA(x0, y, z); FMA(x1, y, z); FMA(x2, y, z); FMA(x3, y, z);
        MFMA_V(acc3, a, b); FMA(x4, y, z); FMA(x5, y, z); FMA(x6, y, z); FMA(x7, y, z);
      }
    } else if constexpr (TEST == T_SPLIT) {
      if ((wave & 4) == 0) {         // wavefronts 0..3: one per SIMD, matrix core only
#pragma unroll
        for (int k = 0; k < 4; ++k) { MFMA_V(acc0, a, b); MFMA_V(acc1, a, b); MFMA_V(acc2, a, b); MFMA_V(acc3, a, b); }
      } else {                       // wavefronts 4..7: the second one of each SIMD, vector ALU only
#pragma unroll
        for (int k = 0; k < 8; ++k) { FMA(x0, y, z); FMA(x1, y, z); FMA(x2, y, z); FMA(x3, y, z); FMA(x4, y, z); FMA(x5, y, z); FMA(x6, y, z); FMA(x7, y, z); }
      }
    } else if constexpr (TEST == T_EXP) {
#pragma unroll
      for (int k = 0; k < 4; ++k) { EXP2(x0); EXP2(x1); EXP2(x2); EXP2(x3); EXP2(x4); EXP2(x5); EXP2(x6); EXP2(x7); }
    } else if constexpr (TEST == T_RCP) {
#pragma unroll
      for (int k = 0; k < 4; ++k) { RCP(x0); RCP(x1); RCP(x2); RCP(x3); RCP(x4); RCP(x5); RCP(x6); RCP(x7); }
    } else if constexpr (TEST == T_MIX_EXP) {
#pragma unroll
      for (int k = 0; k < 4; ++k) { MFMA_V(acc0, a, b); EXP2(x0); MFMA_V(acc1, a, b); EXP2(x1); MFMA_V(acc2, a, b); EXP2(x2); MFMA_V(acc3, a, b); EXP2(x3); }
    } else if constexpr (TEST == T_TANH) {
#pragma unroll
      for (int k = 0; k < 2; ++k) { TANH(x0); TANH(x1); TANH(x2); TANH(x3); TANH(x4); TANH(x5); TANH(x6); TANH(x7); }
    } else if constexpr (TEST == T_LDS_READ) {
      // the wait sits inside the statement: no register of an outstanding read is ever free for the compiler to reuse
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        asm volatile("ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:1024\n ds_read_b128 %2, %8 offset:2048\n ds_read_b128 %3, %8 offset:3072\n"
                     "ds_read_b128 %4, %8 offset:4096\n ds_read_b128 %5, %8 offset:5120\n ds_read_b128 %6, %8 offset:6144\n ds_read_b128 %7, %8 offset:7168\n"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7) : "v"(addr) : "memory");
      }
    } else if constexpr (TEST == T_LDS_CHAIN) {
#pragma unroll
      for (int k = 0; k < 8; ++k) asm volatile("ds_read_b32 %0, %0\n s_waitcnt lgkmcnt(0)" : "+v"(chain));
    } else if constexpr (TEST == T_BARRIER) {
#pragma unroll
      for (int k = 0; k < 8; ++k) __builtin_amdgcn_s_barrier();
    } else if constexpr (TEST == T_EXCHANGE) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        asm volatile("ds_write_b64 %0, %1 offset:32768" :: "v"((uint32_t)(tid * 8)), "v"(*reinterpret_cast<uint64_t*>(&r0)) : "memory");
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("ds_read_b128 %0, %1 offset:32768\n s_waitcnt lgkmcnt(0)" : "=&v"(r1) : "v"(addr) : "memory");
        __builtin_amdgcn_s_barrier();
      }
    }
  }
  asm volatile("s_nop 15\n s_nop 15\n s_nop 15\n s_nop 15\n s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  const uint64_t t1 = now();
  if (blockIdx.x == 0 && tid == 0) *cycles = t1 - t0;
  const float s = acc0.x + acc1.y + acc2.z + acc3.w + x0 + x1 + x2 + x3 + x4 + x5 + x6 + x7 +
                  (float)(r0.x ^ r1.y ^ r2.z ^ r3.w ^ r4.x ^ r5.y ^ r6.z ^ r7.w ^ chain);
  sink[(size_t)blockIdx.x * blockDim.x + tid] = s;
}

struct Spec { const char* name; int threads; int units_per_iter; const char* unit; };
const Spec kSpecs[T_COUNT] = {
    {"mfma_16x16x32_bf16, accumulators in VGPRs, 1 wavefront per SIMD", 256, 16, "MFMA"},
    {"mfma_16x16x32_bf16, accumulators in AGPRs, 1 wavefront per SIMD", 256, 16, "MFMA"},
    {"mfma_16x16x32_bf16, A operand from AGPRs, 1 wavefront per SIMD", 256, 16, "MFMA"},
    {"v_fma_f32, 1 wavefront per SIMD", 256, 32, "FMA"},
    {"1 MFMA + 1 FMA interleaved in one wavefront", 256, 16, "group"},
    {"1 MFMA + 2 FMA interleaved in one wavefront", 256, 16, "group"},
    {"1 MFMA + 4 FMA interleaved in one wavefront", 256, 16, "group"},
    {"2 wavefronts per SIMD: 16 MFMA in one beside 64 FMA in the other", 512, 1, "iteration"},
    {"v_exp_f32", 256, 32, "exp"},
    {"v_rcp_f32", 256, 32, "rcp"},
    {"1 MFMA + 1 v_exp_f32 interleaved in one wavefront", 256, 16, "group"},
    {"tanh = mul, exp, add, rcp, fma", 256, 16, "tanh"},
    {"ds_read_b128, 4 wavefronts of a CU streaming", 256, 32, "read"},
    {"dependent ds_read_b32 (LDS latency)", 256, 8, "read"},
    {"s_barrier, 4 wavefronts", 256, 8, "barrier"},
    {"ds_write_b64 + barrier + ds_read_b128 + barrier (one hand-over)", 256, 4, "hand-over"},
};

// 64 KiB static + 40 KiB dynamic LDS: more than half a CU's 160 KiB, so every workgroup has a CU to itself
constexpr int PAD_LDS_BYTES = 40960;

template <int TEST>
void launch_one(int grid, int threads, int iters, uint64_t* cyc, float* sink, hipStream_t st) {
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(bench_kernel<TEST>), hipFuncAttributeMaxDynamicSharedMemorySize, PAD_LDS_BYTES);
  hipLaunchKernelGGL(bench_kernel<TEST>, dim3(grid), dim3(threads), PAD_LDS_BYTES, st, iters, cyc, sink);
}

template <int TEST>
void dispatch(int which, int grid, int threads, int iters, uint64_t* cyc, float* sink, hipStream_t st) {
  if constexpr (TEST < T_COUNT) {
    if (which == TEST) launch_one<TEST>(grid, threads, iters, cyc, sink, st);
    else dispatch<TEST + 1>(which, grid, threads, iters, cyc, sink, st);
  }
}

}  // namespace

extern "C" {

int es_microbench_count(void) { return T_COUNT; }
const char* es_microbench_name(int which) { return (which >= 0 && which < T_COUNT) ? kSpecs[which].name : ""; }
const char* es_microbench_unit(int which) { return (which >= 0 && which < T_COUNT) ? kSpecs[which].unit : ""; }

// Runs test `which` on every compute unit (one workgroup per CU), `iters` iterations, three times; reports the
// last run: shader-clock cycles per unit of work in one wavefront, milliseconds of the whole launch (HIP
// events), and units of work per second summed over the chip.  Returns 0, or a HIP error code.
int es_microbench_run(int which, int iters, double* cycles_per_unit, double* launch_ms, double* chip_units_per_s) {
  if (which < 0 || which >= T_COUNT || iters < 1 || !cycles_per_unit || !launch_ms || !chip_units_per_s) return -1;
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return (int)e;
  const Spec& sp = kSpecs[which];
  uint64_t* cyc = nullptr;
  float* sink = nullptr;
  if ((e = hipMalloc(&cyc, sizeof(uint64_t))) != hipSuccess) return (int)e;
  if ((e = hipMalloc(&sink, sizeof(float) * (size_t)cus * sp.threads)) != hipSuccess) { (void)hipFree(cyc); return (int)e; }
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  float ms = 0.0f;
  for (int rep = 0; rep < 3; ++rep) {
    (void)hipEventRecord(e0, nullptr);
    dispatch<0>(which, cus, sp.threads, iters, cyc, sink, nullptr);
    (void)hipEventRecord(e1, nullptr);
    e = hipEventSynchronize(e1);
    if (e != hipSuccess) break;
    (void)hipEventElapsedTime(&ms, e0, e1);
  }
  uint64_t c = 0;
  if (e == hipSuccess) e = hipMemcpy(&c, cyc, sizeof(c), hipMemcpyDeviceToHost);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  (void)hipFree(cyc);
  (void)hipFree(sink);
  if (e != hipSuccess) return (int)e;
  const double units_wave = (double)iters * sp.units_per_iter;
  *cycles_per_unit = (double)c / units_wave;
  *launch_ms = ms;
  const double waves = (double)cus * (sp.threads / 64) / (which == T_SPLIT ? 2.0 : 1.0);
  *chip_units_per_s = units_wave * waves / (ms * 1e-3);
  return 0;
}

}  // extern "C"
