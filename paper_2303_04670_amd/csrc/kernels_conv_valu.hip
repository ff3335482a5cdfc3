// Sparse incremental convolution, vector-ALU variant (any k <= 7, stride 1 or 2, any channel
// counts).  Used for the narrow layers, where the per-tile contraction is too thin for the
// matrix cores and the kernel is bound by gathering increments and read-modify-writing z.
//
// Workgroup = one 8 x 8 output tile x 32 output channels, 4 wavefronts.  Lane = output site,
// wavefront = 8 output channels.  Per tile:
//   1. the occupancy words of the input tiles under the halo are staged in LDS; from them each
//      lane decides whether its site is touched; an untouched tile exits at once;
//   2. the input halo patch is gathered into LDS 16 channels at a time; inactive or
//      out-of-image sites are written as zeros without touching global memory (conditioned
//      fetch);
//   3. the weights of one kernel row are staged in LDS; a wave reads its 8 channels with two
//      broadcast ds_read_b128, so each LDS read of an increment feeds 8 FMAs;
//   4. the epilogue read-modify-writes z at touched sites only, forms the activation
//      increment (Eq.12) and ORs the per-site nonzero ballot into the output occupancy word.
#include "evconv_kernels.h"

namespace evk {

namespace {

constexpr int kCpt = 8;     // output channels per wavefront
constexpr int kChunk = 16;  // input channels per LDS pass
constexpr int kChunkPad = 20;

__device__ __forceinline__ float act_f(int act, float v) {
  if (act == kActRelu) return fmaxf(v, 0.0f);
  if (act == kActSigmoid) return 1.0f / (1.0f + expf(-v));
  if (act == kActTanh) return tanhf(v);
  if (act == kActOneMinus) return 1.0f - v;
  return v;
}

__global__ __launch_bounds__(256) void conv_valu_kernel(ConvParams p) {
  const size_t so = (size_t)blockIdx.z * p.st.stride;  // this workgroup's stream
  const float* const in_s = at_stream(p.in, so);
  float* const z_s = at_stream(p.z, so);
  float* const out_s = at_stream(p.out, so);
  extern __shared__ __align__(16) float s_patch[];
  __shared__ uint64_t s_occ[16];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tile = blockIdx.x;
  const int tile_y = tile / p.go.tx, tile_x = tile - tile_y * p.go.tx;
  const int ly = lane >> 3, lx = lane & 7;
  const int oy = tile_y * 8 + ly, ox = tile_x * 8 + lx;
  const bool inb = oy < p.go.h && ox < p.go.w;
  const int s = p.stride, K = p.k;
  const int H = p.gi.h, W = p.gi.w, Cin = p.gi.c, Cout = p.go.c;
  const int iy0 = tile_y * 8 * s - p.pad, ix0 = tile_x * 8 * s - p.pad;  // patch origin (may be < 0)
  const int P = 7 * s + K;                                                // patch edge
  const int rty0 = iy0 >> 3, rtx0 = ix0 >> 3;                             // floor division
  const int rny = ((iy0 + P - 1) >> 3) - rty0 + 1, rnx = ((ix0 + P - 1) >> 3) - rtx0 + 1;

  if (tid < 16) {
    const int ry = tid >> 2, rx = tid & 3;
    const int ty = rty0 + ry, tx = rtx0 + rx;
    uint64_t w = 0;
    if (ry < rny && rx < rnx && ty >= 0 && ty < p.gi.ty && tx >= 0 && tx < p.gi.tx)
      w = p.dense ? ~0ull : at_stream(p.occ_in, so)[ty * p.gi.tx + tx];
    s_occ[tid] = w;
  }
  __syncthreads();

  bool touched = false;
  if (inb) {
    if (p.dense) {
      touched = true;
    } else {
      for (int ky = 0; ky < K; ++ky) {
        const int iy = oy * s - p.pad + ky;
        if ((unsigned)iy >= (unsigned)H) continue;
        for (int kx = 0; kx < K; ++kx) {
          const int ix = ox * s - p.pad + kx;
          if ((unsigned)ix >= (unsigned)W) continue;
          const uint64_t w = s_occ[((iy >> 3) - rty0) * 4 + ((ix >> 3) - rtx0)];
          touched |= (w >> (((iy & 7) << 3) | (ix & 7))) & 1ull;
        }
      }
    }
  }
  const uint64_t touched_word = __ballot(touched);
  if (touched_word == 0) return;  // same word in all four wavefronts

  float acc[kCpt];
#pragma unroll
  for (int j = 0; j < kCpt; ++j) acc[j] = 0.0f;
  const int co0 = blockIdx.y * (4 * kCpt) + wave * kCpt;
  const float* __restrict__ wblock = (const float*)p.w + blockIdx.y * (4 * kCpt);
  float* s_w = s_patch + P * P * kChunkPad;  // staged weights of one kernel row
  const int cop = p.c_out_pad;
  const bool vec_in = (Cin & 3) == 0;

  for (int c0 = 0; c0 < Cin; c0 += kChunk) {
    const int chn = min(kChunk, Cin - c0);
    if (vec_in) {
      const int nv = chn >> 2;
      const int total = P * P * nv;
      for (int e = tid; e < total; e += 256) {
        const int site = e / nv, v = e - site * nv;
        const int py = site / P, px = site - py * P;
        const int iy = iy0 + py, ix = ix0 + px;
        float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
        if ((unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W) {
          const uint64_t w = s_occ[((iy >> 3) - rty0) * 4 + ((ix >> 3) - rtx0)];
          if ((w >> (((iy & 7) << 3) | (ix & 7))) & 1ull)
            val = *(const float4*)&in_s[((size_t)iy * W + ix) * Cin + c0 + v * 4];
        }
        *(float4*)&s_patch[site * kChunkPad + v * 4] = val;
      }
    } else {
      const int total = P * P * chn;
      for (int e = tid; e < total; e += 256) {
        const int site = e / chn, c = e - site * chn;
        const int py = site / P, px = site - py * P;
        const int iy = iy0 + py, ix = ix0 + px;
        float val = 0.0f;
        if ((unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W) {
          const uint64_t w = s_occ[((iy >> 3) - rty0) * 4 + ((ix >> 3) - rtx0)];
          if ((w >> (((iy & 7) << 3) | (ix & 7))) & 1ull) val = in_s[((size_t)iy * W + ix) * Cin + c0 + c];
        }
        s_patch[site * kChunkPad + c] = val;
      }
    }
    // one kernel row at a time: its weights [kx][c][32 channels of this workgroup] are staged in
    // LDS (wave-uniform reads are broadcasts), so the inner loop never waits on memory
    for (int ky = 0; ky < K; ++ky) {
      __syncthreads();  // patch complete (first row) / previous row's weights no longer read
      const int wtotal = K * chn * 32;
      for (int e = tid; e < wtotal; e += 256) {
        const int j = e & 31, rc = e >> 5;
        const int kx = rc / chn, c = rc - kx * chn;
        s_w[e] = wblock[((size_t)(ky * K + kx) * Cin + c0 + c) * cop + j];
      }
      __syncthreads();
      for (int kx = 0; kx < K; ++kx) {
        const float* prow = &s_patch[((ly * s + ky) * P + lx * s + kx) * kChunkPad];
        const float* wrow = &s_w[kx * chn * 32 + wave * kCpt];
        for (int c = 0; c < chn; ++c) {
          const float a = prow[c];
          const float4 w0 = *(const float4*)&wrow[c * 32];
          const float4 w1 = *(const float4*)&wrow[c * 32 + 4];
          acc[0] = fmaf(a, w0.x, acc[0]); acc[1] = fmaf(a, w0.y, acc[1]);
          acc[2] = fmaf(a, w0.z, acc[2]); acc[3] = fmaf(a, w0.w, acc[3]);
          acc[4] = fmaf(a, w1.x, acc[4]); acc[5] = fmaf(a, w1.y, acc[5]);
          acc[6] = fmaf(a, w1.z, acc[6]); acc[7] = fmaf(a, w1.w, acc[7]);
        }
      }
    }
    __syncthreads();
  }

  bool nz = false;
  if (touched) {
    const size_t qoff = ((size_t)oy * p.go.w + ox) * Cout;
#pragma unroll
    for (int j = 0; j < kCpt; ++j) {
      const int co = co0 + j;
      if (co < Cout) {
        float o;
        if (p.dense) {
          const float z = acc[j] + (p.bias ? p.bias[co] : 0.0f);
          z_s[qoff + co] = z;
          o = act_f(p.act, z);
        } else {
          const float z_old = z_s[qoff + co];
          const float z_new = z_old + acc[j];
          z_s[qoff + co] = z_new;
          o = (p.act == kActNone) ? acc[j] : act_f(p.act, z_new) - act_f(p.act, z_old);
        }
        out_s[qoff + co] = o;
        nz |= (o != 0.0f);
      }
    }
  }
  const uint64_t nz_word = p.dense ? touched_word : __ballot(touched && nz);
  if (lane == 0) {
    if (nz_word) atomicOr((unsigned long long*)&at_stream(p.occ_out, so)[tile], (unsigned long long)nz_word);
    if (wave == 0 && blockIdx.y == 0) at_stream(p.occ_touched, so)[tile] = touched_word;
  }
}

}  // namespace

void launch_conv_valu(const ConvParams& p, hipStream_t s) {
  const int P = 7 * p.stride + p.k;
  const size_t lds = ((size_t)P * P * kChunkPad + (size_t)p.k * kChunk * 32) * sizeof(float);
  dim3 grid(p.go.tiles(), (p.go.c + 4 * kCpt - 1) / (4 * kCpt), p.st.n);
  hipLaunchKernelGGL(conv_valu_kernel, grid, dim3(256), lds, s, p);
}

}  // namespace evk
