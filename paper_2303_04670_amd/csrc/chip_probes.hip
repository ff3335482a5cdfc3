// Small timing probes of the properties of the chip that the matrix-core convolution is designed
// around.  Not on any product path: evconv_debug_chip_probes runs them on request (bench.py
// --chip-probes) so that the figures quoted for them can be reproduced.
//
//   1. An fp32 matrix instruction and ordinary vector instructions of the same wave do not overlap.
//   2. Two waves of one SIMD, one issuing fp32 MFMAs and one vector instructions, take the sum of
//      their solo times; with bf16 MFMAs they overlap.
//   3. A wave that walks a chain of dependent global loads (or LDS reads) next to waves that issue
//      MFMAs back to back makes almost no progress until they are done.
//   4. The lanes of one LDS atomic that hit one word are served one after the other (microseconds
//      per instruction), and LDS reads of the other waves of the CU are slowed meanwhile.
//
// Probe kernel: one workgroup of 16 waves fills a CU with four waves per SIMD.  A wave reads the
// SIMD it runs on from the hardware-id register and takes the next free "slot" of that SIMD, so
// slot s is one wave on every SIMD, however the dispatcher dealt the waves.  Every slot is given a
// role and an iteration count; each wave times itself with the 100 MHz wall clock.  Every loop
// has a fixed trip count.
#include <algorithm>
#include <vector>

#include "evconv_kernels.h"

namespace evk {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

enum Role {
  kIdle = 0,
  kMfmaF32,        // dependent chain of v_mfma_f32_32x32x2_f32
  kMfmaBf16,       // dependent chain of v_mfma_f32_32x32x16_bf16
  kValu,           // eight independent v_fma_f32 chains
  kGlobalChain,    // each load's address comes from the previous load
  kLdsChain,       // the same through LDS
  kLdsAtomicSame,  // 64 lanes OR a bit into one LDS word
  kLdsAtomicOwn,   // 64 lanes OR a bit into 64 different words
  kLdsRead,        // independent 16-byte LDS reads
  kMfmaF32Nop,     // the fp32 chain with a 16-cycle s_nop after every MFMA
};

struct ProbeParams {
  int role[4];
  int iters[4];
  const unsigned* chase;        // zero-filled, >= 4 KiB
  unsigned long long* elapsed;  // [workgroup][16 waves], ticks of 10 ns
  float* sink;
};

__global__ __launch_bounds__(1024) void probe_kernel(ProbeParams p) {
  __shared__ unsigned s_words[64];
  __shared__ unsigned s_chain[1024];
  __shared__ __align__(16) float s_buf[4096];
  __shared__ int s_taken[4];
  const int tid = threadIdx.x, lane = tid & 63;
  if (tid < 4) s_taken[tid] = 0;
  if (tid < 64) s_words[tid] = 0;
  s_chain[tid] = (unsigned)((tid * 7 + 3) & 1023);
  for (int i = tid; i < 4096; i += 1024) s_buf[i] = (float)i;
  __syncthreads();
  // HW_ID (register 4), bits 4-5: the SIMD of this wave
  const int simd = (int)__builtin_amdgcn_s_getreg(4 | (4 << 6) | (1 << 11)) & 3;
  int slot = 0;
  if (lane == 0) slot = atomicAdd(&s_taken[simd], 1);
  slot = min(__builtin_amdgcn_readfirstlane(slot), 3);
  __syncthreads();
  const int role = p.role[slot], iters = p.iters[slot];
  float res = 0.0f;
  const unsigned long long t0 = wall_clock64();
  if (role == kMfmaF32) {
    floatx16 acc;
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
    const float a = 1.0f + lane, b = 2.0f;
    for (int it = 0; it < iters; ++it) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
    for (int i = 0; i < 16; ++i) res += acc[i];
  } else if (role == kMfmaF32Nop) {
    floatx16 acc;
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
    const float a = 1.0f + lane, b = 2.0f;
    for (int it = 0; it < iters; ++it) {
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
      asm volatile("s_nop 15");
    }
    for (int i = 0; i < 16; ++i) res += acc[i];
  } else if (role == kMfmaBf16) {
    floatx16 acc;
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(1.0f + i); b[i] = (__bf16)(0.5f * lane); }
    for (int it = 0; it < iters; ++it) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    for (int i = 0; i < 16; ++i) res += acc[i];
  } else if (role == kValu) {
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = tid * 0.001f + i;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int k = 0; k < 8; ++k) x[k] = __builtin_fmaf(x[k], 1.0001f, 0.5f);
    }
    for (int i = 0; i < 8; ++i) res += x[i];
  } else if (role == kGlobalChain) {
    unsigned x = lane;
    for (int it = 0; it < iters; ++it) x = __builtin_nontemporal_load(&p.chase[x & 1023]) & 1023;
    res = (float)x;
  } else if (role == kLdsChain) {
    unsigned x = lane;
    for (int it = 0; it < iters; ++it) x = s_chain[x & 1023];
    res = (float)x;
  } else if (role == kLdsAtomicSame) {
    for (int it = 0; it < iters; ++it) atomicOr(&s_words[0], 1u << (lane & 31));
  } else if (role == kLdsAtomicOwn) {
    for (int it = 0; it < iters; ++it) atomicOr(&s_words[lane], 1u << (it & 31));
  } else if (role == kLdsRead) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int it = 0; it < iters; ++it) {
      const float4 v = *(const float4*)&s_buf[lane * 4 + (it & 15) * 256];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    res = acc.x + acc.y + acc.z + acc.w;
  }
  const unsigned long long t1 = wall_clock64();
  if (lane == 0) p.elapsed[(size_t)blockIdx.x * 16 + slot * 4 + simd] = t1 - t0;
  if (res == 123.456f) p.sink[0] = res + (float)s_words[lane];  // (keeps the loops alive)
}

// one wave per SIMD: one fp32 MFMA plus KV independent vector instructions per iteration
template <int KV>
__global__ __launch_bounds__(256) void same_wave_kernel(float* sink, int iters) {
  floatx16 acc;
  for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
  const float a = 1.0f + threadIdx.x, b = 2.0f;
  float x[8];
  for (int i = 0; i < 8; ++i) x[i] = threadIdx.x * 0.001f + i;
  for (int it = 0; it < iters; ++it) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
#pragma unroll
    for (int k = 0; k < KV; ++k) x[k & 7] = __builtin_fmaf(x[k & 7], 1.0001f, 0.5f);
  }
  float s = 0.0f;
  for (int i = 0; i < 16; ++i) s += acc[i];
  for (int i = 0; i < 8; ++i) s += x[i];
  if (s == 123.456f) sink[0] = s;
}

constexpr int kProbeGroups = 256;

struct ProbeRun {
  hipStream_t stream;
  unsigned* chase;
  unsigned long long* elapsed;
  float* sink;
  // median over the workgroups of the slowest wave of `slot`, in microseconds
  bool run(const int (&role)[4], const int (&iters)[4], float (&slot_us)[4]) {
    ProbeParams p;
    for (int i = 0; i < 4; ++i) { p.role[i] = role[i]; p.iters[i] = iters[i]; }
    p.chase = chase; p.elapsed = elapsed; p.sink = sink;
    for (int rep = 0; rep < 2; ++rep)  // (the first launch warms the instruction cache)
      hipLaunchKernelGGL(probe_kernel, dim3(kProbeGroups), dim3(1024), 0, stream, p);
    std::vector<unsigned long long> h((size_t)kProbeGroups * 16);
    if (hipMemcpyAsync(h.data(), elapsed, h.size() * sizeof(h[0]), hipMemcpyDeviceToHost, stream) != hipSuccess) return false;
    if (hipStreamSynchronize(stream) != hipSuccess) return false;
    for (int s = 0; s < 4; ++s) {
      std::vector<double> v;
      for (int g = 0; g < kProbeGroups; ++g) {
        unsigned long long m = 0;
        for (int w = 0; w < 4; ++w) m = std::max(m, h[(size_t)g * 16 + s * 4 + w]);
        v.push_back((double)m * 0.01);
      }
      std::sort(v.begin(), v.end());
      slot_us[s] = (float)v[v.size() / 2];
    }
    return true;
  }
};

template <int KV>
bool same_wave_cycles(hipStream_t s, float* sink, float& cycles) {
  const int iters = 20000;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return false;
  hipLaunchKernelGGL(same_wave_kernel<KV>, dim3(256), dim3(256), 0, s, sink, iters);
  bool ok = hipEventRecord(e0, s) == hipSuccess;
  hipLaunchKernelGGL(same_wave_kernel<KV>, dim3(256), dim3(256), 0, s, sink, iters);
  ok = ok && hipEventRecord(e1, s) == hipSuccess;
  ok = ok && hipEventSynchronize(e1) == hipSuccess;
  float ms = 0.0f;
  ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  cycles = ms * 1e-3f * 2.4e9f / iters;
  return ok;
}

}  // namespace

// out[0..3]   cycles per iteration (at 2.4 GHz) of one wave per SIMD issuing one fp32 MFMA plus 0, 4, 16, 32
//             independent vector instructions
// out[4..7]   us: vector loop alone, fp32 MFMA chain alone, vector loop beside the chain, chain beside the loop
//             (one wave each on every SIMD)
// out[8..10]  us: bf16 MFMA chain alone, vector loop beside it, chain beside the loop
// out[11..14] us: chain of dependent global loads alone / beside three fp32 MFMA chain waves per SIMD; LDS chain likewise
// out[15..16] ns per LDS atomic instruction: 64 lanes on one word / on 64 words
// out[17..19] us: 16-byte LDS read loop alone / beside same-word atomics of another wave / beside 64-word atomics
// out[20..22] us: fp32 MFMA chain with a 16-cycle s_nop after every MFMA, alone; the global-load chain and the LDS
//             chain beside three such waves per SIMD
int chip_probes(void* scratch, size_t scratch_bytes, hipStream_t s, float* out, int n) {
  if (!scratch || scratch_bytes < kChipProbeScratch || !out || n < kChipProbeValues) return -1;
  launch_fill_u64((uint64_t*)scratch, kChipProbeScratch / 8, 0, Streams{0, 1}, s);
  ProbeRun r;
  r.stream = s;
  r.chase = (unsigned*)scratch;
  r.elapsed = (unsigned long long*)((char*)scratch + 65536);
  r.sink = (float*)((char*)scratch + 32768);
  bool ok = same_wave_cycles<0>(s, r.sink, out[0]) && same_wave_cycles<4>(s, r.sink, out[1]) &&
            same_wave_cycles<16>(s, r.sink, out[2]) && same_wave_cycles<32>(s, r.sink, out[3]);
  float t[4];
  const int kM = 8000, kV = 8000, kB = 16000;  // MFMA chain, vector loop (x 8 instructions), bf16 chain
  ok = ok && r.run({kValu, kIdle, kIdle, kIdle}, {kV, 0, 0, 0}, t); out[4] = t[0];
  ok = ok && r.run({kIdle, kMfmaF32, kIdle, kIdle}, {0, kM, 0, 0}, t); out[5] = t[1];
  ok = ok && r.run({kValu, kMfmaF32, kIdle, kIdle}, {kV, kM, 0, 0}, t); out[6] = t[0]; out[7] = t[1];
  ok = ok && r.run({kIdle, kMfmaBf16, kIdle, kIdle}, {0, kB, 0, 0}, t); out[8] = t[1];
  ok = ok && r.run({kValu, kMfmaBf16, kIdle, kIdle}, {kV, kB, 0, 0}, t); out[9] = t[0]; out[10] = t[1];
  ok = ok && r.run({kGlobalChain, kIdle, kIdle, kIdle}, {100, 0, 0, 0}, t); out[11] = t[0];
  ok = ok && r.run({kGlobalChain, kMfmaF32, kMfmaF32, kMfmaF32}, {100, kM, kM, kM}, t); out[12] = t[0];
  ok = ok && r.run({kLdsChain, kIdle, kIdle, kIdle}, {1000, 0, 0, 0}, t); out[13] = t[0];
  ok = ok && r.run({kLdsChain, kMfmaF32, kMfmaF32, kMfmaF32}, {1000, kM, kM, kM}, t); out[14] = t[0];
  const int kA = 2000, kR = 20000;
  ok = ok && r.run({kLdsAtomicSame, kIdle, kIdle, kIdle}, {kA, 0, 0, 0}, t); out[15] = t[0] * 1000.0f / kA;
  ok = ok && r.run({kLdsAtomicOwn, kIdle, kIdle, kIdle}, {kA, 0, 0, 0}, t); out[16] = t[0] * 1000.0f / kA;
  ok = ok && r.run({kIdle, kLdsRead, kIdle, kIdle}, {0, kR, 0, 0}, t); out[17] = t[1];
  ok = ok && r.run({kLdsAtomicSame, kLdsRead, kIdle, kIdle}, {8 * kA, kR, 0, 0}, t); out[18] = t[1];
  ok = ok && r.run({kLdsAtomicOwn, kLdsRead, kIdle, kIdle}, {8 * kA, kR, 0, 0}, t); out[19] = t[1];
  ok = ok && r.run({kIdle, kMfmaF32Nop, kIdle, kIdle}, {0, kM, 0, 0}, t); out[20] = t[1];
  ok = ok && r.run({kGlobalChain, kMfmaF32Nop, kMfmaF32Nop, kMfmaF32Nop}, {100, kM, kM, kM}, t); out[21] = t[0];
  ok = ok && r.run({kLdsChain, kMfmaF32Nop, kMfmaF32Nop, kMfmaF32Nop}, {1000, kM, kM, kM}, t); out[22] = t[0];
  return ok ? kChipProbeValues : -2;
}

}  // namespace evk
