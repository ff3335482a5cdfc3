// Sparse incremental convolution for narrow inputs, on the matrix cores.
//
// For layers whose whole contraction K = taps x c_in is at most 128 and whose c_out is at least 16
// (the last block of 32 output channels is zero-padded): the first convolution on the event tensor (c_in = 2..5 channels).  With so few input
// channels a per-tap channel contraction is too thin for an MFMA, so the contraction runs over
// the flattened index k = tap * c_in + ci (im2col by addressing, nothing is materialised):
//   A[m][k] = patch[site(m) + tap offset(k)][ci(k)]   one ds_read_b32 through a k -> LDS-offset table
//   B[k][n] = weights re-laid as [KP][c_out] (KP = K rounded up to 16, zero rows beyond K), staged
//             in LDS once per workgroup
// v_mfma_f32_32x32x2_f32, fp32 operands and accumulation (bf16-declared weights are widened, which
// is at least as accurate as the bf16 path).
//
// Workgroup = 32 * NB output channels, walking 8 x 8 output tiles with the grid's stride (the
// weights are staged once); wave = (half tile, 32 channels),
// so every wave owns a whole 32 x 32 accumulator block: no partial sums, and the epilogue goes
// straight from the accumulator registers to memory (register i of lanes 0-31 is one site's 32
// channels = a 128-byte row segment; lanes 32-63 hold the site four further on).
// Masks, conditioned fetch, z read-modify-write, activation increment (Eq.12-14) and occupancy
// words as in the other convolution kernels.
#include <algorithm>

#include "evconv_kernels.h"

namespace evk {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kMaxK = 128;  // largest padded contraction length

__device__ __forceinline__ float act_n(int act, float v) {
  if (act == kActRelu) return fmaxf(v, 0.0f);
  if (act == kActSigmoid) return 1.0f / (1.0f + expf(-v));
  if (act == kActTanh) return tanhf(v);
  if (act == kActOneMinus) return 1.0f - v;
  return v;
}

template <int NB>
__global__ __launch_bounds__(128 * NB) void conv_narrow_kernel(ConvParams p) {
  const size_t so = (size_t)blockIdx.z * p.st.stride;  // this workgroup's stream
  constexpr int NT = 128 * NB;
  constexpr int NC = 32 * NB;  // output channels per workgroup
  extern __shared__ __align__(16) float s_dyn[];  // [KP][NC] weights, then the patch
  __shared__ uint64_t s_occ[16];
  __shared__ unsigned s_rows[24];
  __shared__ int s_koff[kMaxK];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = wave & 1, nsub = wave >> 1;
  const int s = p.stride, K = p.k;
  const int H = p.gi.h, W = p.gi.w, Cin = p.gi.c, Cout = p.go.c;
  const int P = 7 * s + K;  // patch edge, <= 21
  const int CS = Cin | 1;   // odd LDS site stride
  const int k_tot = K * K * Cin, KP = (k_tot + 15) & ~15;
  float* const s_w = s_dyn;
  float* const s_patch = s_dyn + KP * NC;
  const int cin_magic = (65536 + Cin - 1) / Cin;  // e / Cin == (e * cin_magic) >> 16 for e < 2206 (Cin <= 8)
  const int p_magic = (65536 + P - 1) / P;        // site / P likewise for site < 441

  // once per workgroup: k -> LDS offset of the patch element it reads (relative to the output
  // site's patch origin), and the weights of this workgroup's channels
  for (int k = tid; k < KP; k += NT) {
    int off = 0;
    if (k < k_tot) {
      const int tap = k / Cin, ci = k - tap * Cin;
      const int ky = tap / K, kx = tap - ky * K;
      off = (ky * P + kx) * CS + ci;
    }
    s_koff[k] = off;
  }
  // The weights are fetched when the first touched tile is met (a workgroup without one leaves
  // without reading them), all of a thread's share at once and between that tile's z and patch
  // requests, so that one memory latency covers the three.
  const float4* __restrict__ wsrc = (const float4*)((const float*)p.w + blockIdx.y * NC);
  constexpr int NC4 = NC / 4;
  constexpr int WV = kMaxK * NC4 / NT;  // float4 of weights per thread (8)
  bool staged = false;

  // workgroups walk the tiles with the grid's stride; the weights stay in LDS
  for (int tile = blockIdx.x; tile < p.go.tiles(); tile += gridDim.x) {
  const int tile_y = tile / p.go.tx, tile_x = tile - tile_y * p.go.tx;
  const int iy0 = tile_y * 8 * s - p.pad, ix0 = tile_x * 8 * s - p.pad;
  const int rty0 = iy0 >> 3, rtx0 = ix0 >> 3;
  const int rny = ((iy0 + P - 1) >> 3) - rty0 + 1, rnx = ((ix0 + P - 1) >> 3) - rtx0 + 1;
  __syncthreads();  // the previous tile's masks and patch are no longer in use
  if (tid < 16) {
    const int ry = tid >> 2, rx = tid & 3;
    const int ty = rty0 + ry, tx = rtx0 + rx;
    uint64_t w = 0;
    if (ry < rny && rx < rnx && ty >= 0 && ty < p.gi.ty && tx >= 0 && tx < p.gi.tx)
      w = p.dense ? ~0ull : at_stream(p.occ_in, so)[ty * p.gi.tx + tx];
    s_occ[tid] = w;
  }
  __syncthreads();
  if (tid < P) {  // one bit row per patch row; out-of-image sites are 0
    const int iy = iy0 + tid;
    unsigned bits = 0;
    if ((unsigned)iy < (unsigned)H) {
      const int ry = (iy >> 3) - rty0;
      uint64_t span = 0;
#pragma unroll
      for (int rx = 0; rx < 4; ++rx) span |= ((s_occ[ry * 4 + rx] >> ((iy & 7) * 8)) & 0xffull) << (8 * rx);
      bits = (unsigned)(span >> (ix0 - rtx0 * 8));
      const int lo = max(0, -ix0), hi = min(P, W - ix0);  // valid px in [lo, hi)
      unsigned m = hi >= 32 ? ~0u : ((1u << max(hi, 0)) - 1u);
      m &= ~((1u << lo) - 1u);
      bits &= m;
    }
    s_rows[tid] = bits;
  }
  __syncthreads();

  uint64_t touched_word;  // whole tile, identical in all waves
  {
    const int ly = lane >> 3, lx = lane & 7;
    const int oy = tile_y * 8 + ly, ox = tile_x * 8 + lx;
    bool touched = false;
    if (oy < p.go.h && ox < p.go.w) {
      unsigned rows = 0;
      for (int ky = 0; ky < K; ++ky) rows |= s_rows[ly * s + ky];
      touched = p.dense || ((rows >> (lx * s)) & ((1u << K) - 1u)) != 0;
    }
    touched_word = __ballot(touched);
  }
  if (touched_word == 0) continue;
  const unsigned my_touched = (unsigned)(touched_word >> (32 * half));  // this wave's 32 sites

  // accumulator element (register i, lane l) = local site 8*(i/4) + 4*(l/32) + i%4, channel l%32
  const int co = blockIdx.y * NC + nsub * 32 + (lane & 31);
  const int hi4 = (lane >> 5) * 4;
  float z_old[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int ls = 8 * (i >> 2) + hi4 + (i & 3);
    z_old[i] = 0.0f;
    if (!p.dense && co < Cout && ((my_touched >> ls) & 1u)) {
      const int site = half * 32 + ls;
      const int oy = tile_y * 8 + (site >> 3), ox = tile_x * 8 + (site & 7);
      z_old[i] = at_stream(p.z, so)[((size_t)oy * p.go.w + ox) * Cout + co];
    }
  }

  float4 wreg[WV];
  if (!staged) {
#pragma unroll
    for (int j = 0; j < WV; ++j) {
      const int e = tid + j * NT;
      const int k = e / NC4, n4 = e - k * NC4;
      wreg[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (e < KP * NC4) wreg[j] = wsrc[(size_t)k * (p.c_out_pad / 4) + n4];
    }
  }

  // patch: conditioned fetch, inactive and out-of-image sites become zeros without a memory access
  {
    const __amdgpu_buffer_rsrc_t in_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)at_stream(p.in, so), 0, H * W * Cin * 4, 0x00020000);
    const int total = P * P * Cin;
#pragma unroll 4
    for (int e = tid; e < total; e += NT) {
      const int site = (e * cin_magic) >> 16, c = e - site * Cin;
      const int py = (site * p_magic) >> 16, px = site - py * P;
      unsigned off = 0x80000000u;
      if ((s_rows[py] >> px) & 1u) off = (unsigned)((((iy0 + py) * W + ix0 + px) * Cin + c) * 4);
      s_patch[site * CS + c] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(in_rsrc, off, 0, 0));
    }
  }
  if (!staged) {
#pragma unroll
    for (int j = 0; j < WV; ++j) {
      const int e = tid + j * NT;
      const int k = e / NC4, n4 = e - k * NC4;
      if (e < KP * NC4) *(float4*)&s_w[k * NC + n4 * 4] = wreg[j];
    }
    staged = true;
  }
  __syncthreads();

  floatx16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
  {
    const int m = lane & 31, kh = lane >> 5;
    const int my = half * 4 + (m >> 3), mx = m & 7;
    const float* ap = s_patch + (my * s * P + mx * s) * CS;
    const float* bp = s_w + nsub * 32 + m;
    // blocks of 8 MFMA steps: the table look-ups, then the operand reads, then the MFMAs, so that
    // the LDS latencies of a block overlap instead of forming one chain per step
    for (int k0 = kh; k0 < KP; k0 += 16) {
      const bool full = k0 - kh + 16 <= k_tot;  // (uniform) every k of this block is a real one
      int ko[8];
      float a[8], b[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) ko[j] = s_koff[k0 + 2 * j];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        // (beyond taps x c_in the operand is an explicit zero, not a patch element times a zero
        // weight: the element may be infinite or NaN)
        a[j] = (full || k0 + 2 * j < k_tot) ? ap[ko[j]] : 0.0f;
        b[j] = bp[(k0 + 2 * j) * NC];
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b[j], acc, 0, 0, 0);
    }
  }

  // epilogue straight from the accumulator registers
  unsigned nz = 0;  // nonzero output sites of this wave (bits of its 32-site half)
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int ls = 8 * (i >> 2) + hi4 + (i & 3);
    const bool on = ((my_touched >> ls) & 1u) && co < Cout;  // (c_out rounded up to 32: surplus lanes own nothing)
    float o = 0.0f;
    if (on) {
      const int site = half * 32 + ls;
      const int oy = tile_y * 8 + (site >> 3), ox = tile_x * 8 + (site & 7);
      const size_t q = ((size_t)oy * p.go.w + ox) * Cout + co;
      const float v = acc[i];
      if (p.dense) {
        const float z = v + (p.bias ? p.bias[co] : 0.0f);
        at_stream(p.z, so)[q] = z;
        o = act_n(p.act, z);
      } else {
        const float z_new = z_old[i] + v;
        at_stream(p.z, so)[q] = z_new;
        o = (p.act == kActNone) ? v : act_n(p.act, z_new) - act_n(p.act, z_old[i]);
      }
      at_stream(p.out, so)[q] = o;
    }
    const uint64_t b = __ballot(on && o != 0.0f);
    const int ls_lo = 8 * (i >> 2) + (i & 3);
    if ((unsigned)b) nz |= 1u << ls_lo;
    if ((unsigned)(b >> 32)) nz |= 1u << (ls_lo + 4);
  }
  if (lane == 0) {
    const uint64_t mine = (uint64_t)(p.dense ? my_touched : nz) << (32 * half);
    if (mine) atomicOr((unsigned long long*)&at_stream(p.occ_out, so)[tile], (unsigned long long)mine);  // pre-zeroed word
    if (blockIdx.y == 0 && nsub == 0) {
      const uint64_t t = (uint64_t)my_touched << (32 * half);
      if (t) atomicOr((unsigned long long*)&at_stream(p.occ_touched, so)[tile], (unsigned long long)t);
    }
  }
  }  // tiles
}

}  // namespace

bool conv_narrow_supported(const ConvParams& p) {
  const int k_tot = p.k * p.k * p.gi.c;
  return k_tot <= kMaxK && p.gi.c <= 8 && p.go.c >= 16 && p.c_out_pad == (p.go.c + 31) / 32 * 32 && p.n_fused == 0 &&
         (long long)p.gi.h * p.gi.w * p.gi.c * 4 < (1ll << 31);  // byte offsets of the gather fit 31 bits
}

int conv_narrow_padded_k(int k_tot) { return (k_tot + 15) & ~15; }

void launch_conv_narrow(const ConvParams& p, hipStream_t s) {
  const int P = 7 * p.stride + p.k;
  const int KP = conv_narrow_padded_k(p.k * p.k * p.gi.c);
  const int nb = (p.c_out_pad % 64 == 0) ? 2 : 1;
  const size_t lds = ((size_t)KP * 32 * nb + (size_t)P * P * (p.gi.c | 1)) * sizeof(float);
  // workgroups walk the tiles with the grid's stride; enough of them to fill the chip's resident
  // slots (a tile is one chain of dependent memory round trips, so few long walks are slow)
  dim3 grid(std::min(p.go.tiles(), std::max(4096 / p.st.n, 256)), p.c_out_pad / (32 * nb), p.st.n);
  if (nb == 2) hipLaunchKernelGGL(conv_narrow_kernel<2>, grid, dim3(256), lds, s, p);
  else hipLaunchKernelGGL(conv_narrow_kernel<1>, grid, dim3(128), lds, s, p);
}

}  // namespace evk
