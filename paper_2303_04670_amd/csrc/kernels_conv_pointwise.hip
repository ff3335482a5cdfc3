// 1 x 1 convolutions with few output channels (prediction heads: c_out <= 8, stride 1, no
// padding) and LINEAR on a 1 x 1 grid (classifier).  Both are dot products per site, bound by
// reading the input increment: the matrix-core tiling (32 output channels per block) and the
// general vector kernel (a halo patch through LDS) would waste nearly all of their work here.
//
// conv_pointwise_few_kernel: workgroup = one 8 x 8 tile, four lanes per site.  Lane q of a site
//   reads the float4 channel groups q, q+4, q+8, ... of its site (the four lanes of a site read
//   64 contiguous bytes per step), multiplies by the matching weights [c_out][c_in] and the four
//   partial sums are added with two lane shuffles, in a fixed order.  T = S_in (Eq.13: a 1 x 1
//   window has no footprint); z read-modify-write, activation increment (Eq.12-14), occupancy
//   words as in the other convolution kernels.
// linear_site_kernel: one wavefront per output channel of the single site.
#include "evconv_kernels.h"

namespace evk {

namespace {

constexpr int kMaxFew = 8;  // output channels of the few-channel kernel

__device__ __forceinline__ float act_p(int act, float v) {
  if (act == kActRelu) return fmaxf(v, 0.0f);
  if (act == kActSigmoid) return 1.0f / (1.0f + expf(-v));
  if (act == kActTanh) return tanhf(v);
  if (act == kActOneMinus) return 1.0f - v;
  return v;
}

// z read-modify-write and output increment of one (site, channel) element
__device__ __forceinline__ float finish_element(const ConvParams& p, float* z, float* out, size_t q, int co, float v) {
  float o;
  if (p.dense) {
    const float zn = v + (p.bias ? p.bias[co] : 0.0f);
    z[q] = zn;
    o = act_p(p.act, zn);
  } else {
    const float z_old = z[q];
    const float z_new = z_old + v;
    z[q] = z_new;
    o = (p.act == kActNone) ? v : act_p(p.act, z_new) - act_p(p.act, z_old);
  }
  out[q] = o;
  return o;
}

__global__ __launch_bounds__(256) void conv_pointwise_few_kernel(ConvParams p) {
  __shared__ unsigned s_nz[2];
  const size_t so = (size_t)blockIdx.z * p.st.stride;  // this workgroup's stream
  const int tid = threadIdx.x;
  const int tile = blockIdx.x;
  const int tile_y = tile / p.go.tx, tile_x = tile - tile_y * p.go.tx;
  const int site = tid >> 2, q4 = tid & 3;  // site inside the tile, lane inside the site's group of four
  const int oy = tile_y * 8 + (site >> 3), ox = tile_x * 8 + (site & 7);
  const bool inb = oy < p.go.h && ox < p.go.w;
  const int Cin = p.gi.c, Cout = p.go.c;
  // same geometry in and out: the touched word is the input's occupancy word
  const uint64_t word = p.dense ? ~0ull : at_stream(p.occ_in, so)[tile];
  const bool on = inb && ((word >> site) & 1ull);
  if (tid < 2) s_nz[tid] = 0;
  // all 256 threads see the same word (one broadcast load each); nothing to do for an empty tile
  uint64_t touched_word = 0;
  {
    // in-bounds mask of the tile, so that dense mode and ragged borders agree with `on`
    const int rows = min(8, p.go.h - tile_y * 8), cols = min(8, p.go.w - tile_x * 8);
    const uint64_t rowbits = cols >= 8 ? 0xffull : ((1ull << cols) - 1ull);
    uint64_t m = 0;
    for (int r = 0; r < rows; ++r) m |= rowbits << (8 * r);
    touched_word = word & m;
  }
  // output node kept by this kernel: public tensors are C x H x W
  const int hw = p.go.h * p.go.w;
  float* const pub_y = p.y ? at_stream(p.y, so) : nullptr;
  float* const pub_dy = p.dy ? at_stream(p.dy, so) : nullptr;
  if (touched_word == 0) {
    // nothing changed under this tile: the increment of its sites is zero
    if (pub_dy && inb && q4 == 0)
      for (int j = 0; j < Cout; ++j) pub_dy[(size_t)j * hw + oy * p.go.w + ox] = 0.0f;
    return;
  }
  __syncthreads();

  float acc[kMaxFew];
#pragma unroll
  for (int j = 0; j < kMaxFew; ++j) acc[j] = 0.0f;
  if (on) {
    const float* __restrict__ x = at_stream(p.in, so) + ((size_t)oy * p.gi.w + ox) * Cin;
    const float* __restrict__ w = (const float*)p.w;  // [c_out][c_in]
    if ((Cin & 3) == 0) {
      for (int c = q4 * 4; c < Cin; c += 16) {
        const float4 xv = *(const float4*)&x[c];
#pragma unroll
        for (int j = 0; j < kMaxFew; ++j) {
          if (j >= Cout) break;
          const float4 wv = *(const float4*)&w[(size_t)j * Cin + c];
          acc[j] = fmaf(xv.x, wv.x, acc[j]);
          acc[j] = fmaf(xv.y, wv.y, acc[j]);
          acc[j] = fmaf(xv.z, wv.z, acc[j]);
          acc[j] = fmaf(xv.w, wv.w, acc[j]);
        }
      }
    } else {
      for (int c = q4; c < Cin; c += 4) {
        const float xv = x[c];
#pragma unroll
        for (int j = 0; j < kMaxFew; ++j) {
          if (j >= Cout) break;
          acc[j] = fmaf(xv, w[(size_t)j * Cin + c], acc[j]);
        }
      }
    }
  }
  // add the four lanes of a site: (0 + 1) + (2 + 3), every lane ends with the full sum
#pragma unroll
  for (int j = 0; j < kMaxFew; ++j) {
    acc[j] += __shfl_xor(acc[j], 1);
    acc[j] += __shfl_xor(acc[j], 2);
  }
  bool nz = false;
  if (inb && q4 == 0) {
    float* z = at_stream(p.z, so);
    float* out = at_stream(p.out, so);
    const size_t q0 = ((size_t)oy * p.go.w + ox) * Cout;
#pragma unroll
    for (int j = 0; j < kMaxFew; ++j) {
      if (j >= Cout) break;
      float o = 0.0f;
      if (on) {
        o = finish_element(p, z, out, q0 + j, j, acc[j]);
        nz |= o != 0.0f;
      }
      if (pub_y) {  // the step's output and its increment, as the stand-alone integration writes them
        const size_t e = (size_t)j * hw + oy * p.go.w + ox;
        if (p.int_mode == kIntStep) {
          if (on) pub_y[e] += o;
          pub_dy[e] = o;
        } else if (p.int_mode == kIntReset) {
          pub_y[e] = o;
          pub_dy[e] = 0.0f;
        } else {
          pub_dy[e] = o - pub_y[e];
          pub_y[e] = o;
        }
      }
    }
  }
  if (nz) atomicOr(&s_nz[site >> 5], 1u << (site & 31));
  __syncthreads();
  if (tid == 0) {
    const uint64_t s_out = p.dense ? touched_word : ((uint64_t)s_nz[0] | ((uint64_t)s_nz[1] << 32));
    at_stream(p.occ_out, so)[tile] = s_out;       // this workgroup is the tile's only writer
    at_stream(p.occ_touched, so)[tile] = touched_word;
  }
}

// one wavefront per output channel: the lanes stride through c_in (coalesced weight row), then a
// butterfly adds the 64 partial sums in a fixed order
__global__ __launch_bounds__(256) void linear_site_kernel(ConvParams p) {
  const size_t so = (size_t)blockIdx.z * p.st.stride;
  const int lane = threadIdx.x & 63;
  const int co = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int Cin = p.gi.c, Cout = p.go.c;
  const bool active = p.dense || (at_stream(p.occ_in, so)[0] & 1ull);
  if (!active || co >= Cout) return;  // uniform per wavefront
  const float* __restrict__ x = at_stream(p.in, so);
  const float* __restrict__ w = (const float*)p.w + (size_t)co * Cin;  // [c_out][c_in]
  float acc = 0.0f;
  for (int c = lane; c < Cin; c += 64) acc = fmaf(x[c], w[c], acc);
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) acc += __shfl_xor(acc, m);
  if (lane == 0) {
    const bool nz = finish_element(p, at_stream(p.z, so), at_stream(p.out, so), (size_t)co, co, acc) != 0.0f;
    // pre-zeroed words; the wavefronts of one launch OR their share in
    if (p.dense || nz) atomicOr((unsigned long long*)at_stream(p.occ_out, so), 1ull);
    if (co == 0) at_stream(p.occ_touched, so)[0] = 1ull;
  }
}

}  // namespace

bool conv_pointwise_integrates(const ConvParams& p) { return !(p.go.h == 1 && p.go.w == 1 && p.go.c > kMaxFew); }

bool conv_pointwise_supported(const ConvParams& p) {
  if (p.k != 1 || p.stride != 1 || p.pad != 0 || p.n_fused != 0) return false;
  if (p.gi.h != p.go.h || p.gi.w != p.go.w) return false;
  return p.go.c <= kMaxFew || (p.go.h == 1 && p.go.w == 1);
}

void launch_conv_pointwise(const ConvParams& p, hipStream_t s) {
  if (p.go.h == 1 && p.go.w == 1 && p.go.c > kMaxFew)
    hipLaunchKernelGGL(linear_site_kernel, dim3((p.go.c + 3) / 4, 1, p.st.n), dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL(conv_pointwise_few_kernel, dim3(p.go.tiles(), 1, p.st.n), dim3(256), 0, s, p);
}

}  // namespace evk
