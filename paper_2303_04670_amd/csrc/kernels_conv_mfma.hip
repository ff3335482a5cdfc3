// Sparse incremental convolution on the matrix cores, fp32 (v_mfma_f32_32x32x2_f32).
//
// Used where the per-tile channel contraction is a dense GEMM: c_in % 16 == 0, c_out % 32 == 0.
// Implicit GEMM per touched output tile: M = 64 sites (two 32-row blocks: tile rows 0-3 and
// 4-7), N = 32 output channels per workgroup, K = taps x c_in.
//
// Workgroup = NW (4 or 8) wavefronts that split K: the (tap, 8-channel group) units of every
// channel chunk are dealt round-robin to the waves; each wave keeps both 32 x 32 accumulators
// (32 VGPRs) and the partial sums are added through LDS at the end.  K-splitting (rather than
// N-splitting) is what fills the chip on the low-resolution layers, where a layer has only
// 24-88 tiles; those layers run with 8 waves.
//   A operand: the input halo patch of the current chunk, gathered once per workgroup into LDS
//     (zeros for inactive / out-of-image sites, which are never fetched).  The next chunk's
//     patch is fetched into registers while the current one is being contracted.  A lane
//     reads 4 consecutive channels of its site with one ds_read_b128.
//   B operand: weights re-laid as [tap][c_in/4][c_out][4] so that a lane's 4 channels of its
//     output column are one 16-byte global load (L2-resident), prefetched two units ahead.
//   K order inside an 8-channel group: MFMA j contracts channels {j, 4+j}; lanes 0-31 hold
//     channel j, lanes 32-63 channel 4+j, for both operands.
// Epilogue: lane = output channel, so every z / increment access is a 128-byte row segment.
#include "evconv_kernels.h"

namespace evk {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float act_m(int act, float v) {
  if (act == kActRelu) return fmaxf(v, 0.0f);
  if (act == kActSigmoid) return 1.0f / (1.0f + expf(-v));
  return v;
}

// largest halo patch: 32-channel chunks are used with stride 1 only (14 x 14 for 7 x 7 taps),
// 16-channel chunks also with stride 2 (21 x 21)
constexpr int max_patch_sites(int chunk) { return chunk == 32 ? 14 * 14 : 21 * 21; }

template <int CHUNK, int NW>
__global__ __launch_bounds__(NW * 64) void conv_mfma_f32_kernel(ConvParams p) {
  constexpr int NT = NW * 64;
  constexpr int CS = CHUNK + 4;  // LDS site stride in floats: CS/4 odd => conflict-free b128 reads
  constexpr int KG = CHUNK / 8;  // 8-channel groups per chunk
  constexpr int NV = CHUNK / 4;  // float4 per patch site
  constexpr int MAXV = (max_patch_sites(CHUNK) * NV + NT - 1) / NT;  // patch float4 per thread, upper bound
  extern __shared__ __align__(16) float s_mem[];
  __shared__ uint64_t s_occ[16];
  __shared__ unsigned s_nz[2];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tile = blockIdx.x;
  const int tile_y = tile / p.go.tx, tile_x = tile - tile_y * p.go.tx;
  const int s = p.stride, K = p.k;
  const int H = p.gi.h, W = p.gi.w, Cin = p.gi.c, Cout = p.go.c;
  const int iy0 = tile_y * 8 * s - p.pad, ix0 = tile_x * 8 * s - p.pad;
  const int P = 7 * s + K;
  const int rty0 = iy0 >> 3, rtx0 = ix0 >> 3;
  const int rny = ((iy0 + P - 1) >> 3) - rty0 + 1, rnx = ((ix0 + P - 1) >> 3) - rtx0 + 1;

  if (tid < 16) {
    const int ry = tid >> 2, rx = tid & 3;
    const int ty = rty0 + ry, tx = rtx0 + rx;
    uint64_t w = 0;
    if (ry < rny && rx < rnx && ty >= 0 && ty < p.gi.ty && tx >= 0 && tx < p.gi.tx)
      w = p.dense ? ~0ull : p.occ_in[ty * p.gi.tx + tx];
    s_occ[tid] = w;
  }
  if (tid < 2) s_nz[tid] = 0;
  __syncthreads();

  // touched word of the tile (identical in all waves)
  uint64_t touched_word;
  {
    const int oy = tile_y * 8 + (lane >> 3), ox = tile_x * 8 + (lane & 7);
    bool touched = false;
    if (oy < p.go.h && ox < p.go.w) {
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
    touched_word = __ballot(touched);
  }
  if (touched_word == 0) return;

  // ---- patch gather: per thread a fixed list of (LDS offset, byte offset into the input).
  // Inactive and out-of-image sites get an offset beyond the buffer: the hardware bounds check
  // of the buffer load returns zeros for them without touching memory (conditioned fetch).
  constexpr unsigned kOob = 0x80000000u;
  const int total_v = P * P * NV;
  int lds_off[MAXV];
  unsigned g_off[MAXV];
#pragma unroll
  for (int j = 0; j < MAXV; ++j) {
    const int e = tid + j * NT;
    lds_off[j] = -1;
    g_off[j] = kOob;
    if (e < total_v) {
      const int site = e / NV, v = e - site * NV;
      const int py = site / P, px = site - py * P;
      const int iy = iy0 + py, ix = ix0 + px;
      lds_off[j] = site * CS + v * 4;
      if ((unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W) {
        const uint64_t w = s_occ[((iy >> 3) - rty0) * 4 + ((ix >> 3) - rtx0)];
        if ((w >> (((iy & 7) << 3) | (ix & 7))) & 1ull) g_off[j] = (unsigned)(((iy * W + ix) * Cin + v * 4) * 4);
      }
    }
  }
  const __amdgpu_buffer_rsrc_t in_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.in, 0, H * W * Cin * 4, 0x00020000);
  float4 pre[MAXV];
  auto fetch = [&](int c0) {
#pragma unroll
    for (int j = 0; j < MAXV; ++j)
      pre[j] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(in_rsrc, g_off[j], c0 * 4, 0));
  };
  auto stash = [&]() {
#pragma unroll
    for (int j = 0; j < MAXV; ++j)
      if (lds_off[j] >= 0) *(float4*)&s_mem[lds_off[j]] = pre[j];
  };

  floatx16 acc0, acc1;
#pragma unroll
  for (int i = 0; i < 16; ++i) { acc0[i] = 0.0f; acc1[i] = 0.0f; }
  const int half = lane >> 5, m = lane & 31;
  const int mly = m >> 3, mlx = m & 7;  // site of this lane inside a 32-row block
  const int co0 = blockIdx.y * 32;
  const int cop = p.c_out_pad;
  const int n_units = K * K * KG;
  const int cin4 = Cin >> 2;
  const int a_lane_off = (mly * s * P + mlx * s) * CS + half * 4;
  const int a_blk1 = 4 * s * P * CS;
  const float4* __restrict__ wlane = (const float4*)p.w + (size_t)half * cop + co0 + m;
  // units of this wave: u_j = wave + j * NW, j < n_mine
  const int n_mine = (n_units - wave + NW - 1) / NW;
  const int last = n_mine - 1;
  const int k_magic = (65536 + K - 1) / K;  // tap / K == (tap * k_magic) >> 16 for tap < 49

  fetch(0);
  for (int c0 = 0; c0 < Cin; c0 += CHUNK) {
    __syncthreads();  // all waves are done reading the previous chunk
    stash();
    __syncthreads();
    if (n_mine <= 0) {  // more waves than units (1 x 1 taps): only help with the gather
      if (c0 + CHUNK < Cin) fetch(c0 + CHUNK);
      continue;
    }
    const float4* wchunk = wlane + (size_t)(c0 >> 2) * cop;
    // unit j -> LDS offset of its A fragment and address of its B fragment (clamped to the last
    // unit so that look-ahead loads stay unconditional and in bounds)
    auto b_ptr = [&](int j) {
      const int u = wave + min(j, last) * NW;
      const int tap = u / KG, kg = u % KG;
      return wchunk + ((size_t)tap * cin4 + kg * 2) * cop;
    };
    auto a_off = [&](int j) {
      const int u = wave + j * NW;
      const int tap = u / KG, kg = u % KG;
      const int ky = (tap * k_magic) >> 16, kx = tap - ky * K;
      return a_lane_off + (ky * P + kx) * CS + kg * 8;
    };
    auto unit = [&](int j, const float4& b) {
      const float* ap = &s_mem[a_off(j)];
      const float4 a0 = *(const float4*)ap;
      const float4 a1 = *(const float4*)(ap + a_blk1);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.x, b.x, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.x, b.x, acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.y, b.y, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.y, b.y, acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.z, b.z, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.z, b.z, acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.w, b.w, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.w, b.w, acc1, 0, 0, 0);
    };
    // ring of three weight fragments, two units of look-ahead, no register copies: vector loads
    // complete in order, so each wait only covers loads issued two units earlier
    float4 bq0 = *b_ptr(0);
    float4 bq1 = *b_ptr(1);
    float4 bq2;
    if (c0 + CHUNK < Cin) fetch(c0 + CHUNK);  // next chunk's patch, in flight during the contraction
    int j = 0;
    for (; j + 3 <= n_mine; j += 3) {
      bq2 = *b_ptr(j + 2);
      unit(j, bq0);
      bq0 = *b_ptr(j + 3);
      unit(j + 1, bq1);
      bq1 = *b_ptr(j + 4);
      unit(j + 2, bq2);
    }
    if (j < n_mine) unit(j, bq0);
    if (j + 1 < n_mine) unit(j + 1, bq1);
  }
  // ---- reduce the NW partial sums through LDS: slots [4][block*16 + reg][lane]
  __syncthreads();
  if (NW == 8) {
    if (wave >= 4) {
      float* part = s_mem + (wave - 4) * (32 * 64);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        part[i * 64 + lane] = acc0[i];
        part[(16 + i) * 64 + lane] = acc1[i];
      }
    }
    __syncthreads();
    if (wave < 4) {
      const float* part = s_mem + wave * (32 * 64);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        acc0[i] += part[i * 64 + lane];
        acc1[i] += part[(16 + i) * 64 + lane];
      }
    }
  }
  if (wave < 4) {
    float* part = s_mem + wave * (32 * 64);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      part[i * 64 + lane] = acc0[i];
      part[(16 + i) * 64 + lane] = acc1[i];
    }
  }
  __syncthreads();

  // epilogue: thread -> (output channel = tid % 32, 64 / (NT / 32) sites); accumulator element
  // (block b, register i, lane l) is site b*32 + 8*(i/4) + 4*(l/32) + i%4, channel l%32
  const int co = tid & 31;
  uint64_t nz_sites = 0;
  constexpr int SITES_PER_IT = NT / 32;
  for (int it = 0; it < 64 / SITES_PER_IT; ++it) {
    const int site = it * SITES_PER_IT + (tid >> 5);
    if (!((touched_word >> site) & 1ull)) continue;
    const int b = site >> 5, r = site & 31;
    const int reg = (r >> 3) * 4 + (r & 3);
    const int l = ((r >> 2) & 1) * 32 + co;
    const int off = (b * 16 + reg) * 64 + l;
    const float v = (s_mem[off] + s_mem[off + 2048]) + (s_mem[off + 4096] + s_mem[off + 6144]);
    const int oy = tile_y * 8 + (site >> 3), ox = tile_x * 8 + (site & 7);
    const size_t q = ((size_t)oy * p.go.w + ox) * Cout + co0 + co;
    float o;
    if (p.dense) {
      const float z = v + (p.bias ? p.bias[co0 + co] : 0.0f);
      p.z[q] = z;
      o = act_m(p.act, z);
    } else {
      const float z_old = p.z[q];
      const float z_new = z_old + v;
      p.z[q] = z_new;
      o = (p.act == kActNone) ? v : act_m(p.act, z_new) - act_m(p.act, z_old);
    }
    p.out[q] = o;
    if (o != 0.0f) nz_sites |= 1ull << site;
  }
  if (!p.dense) {
    if (nz_sites) {
      if ((unsigned)nz_sites) atomicOr(&s_nz[0], (unsigned)nz_sites);
      if ((unsigned)(nz_sites >> 32)) atomicOr(&s_nz[1], (unsigned)(nz_sites >> 32));
    }
    __syncthreads();
    if (tid == 0) {
      const uint64_t w = (uint64_t)s_nz[0] | ((uint64_t)s_nz[1] << 32);
      if (w) atomicOr((unsigned long long*)&p.occ_out[tile], (unsigned long long)w);
      if (blockIdx.y == 0) p.occ_touched[tile] = touched_word;
    }
  } else if (tid == 0) {
    atomicOr((unsigned long long*)&p.occ_out[tile], (unsigned long long)touched_word);
    if (blockIdx.y == 0) p.occ_touched[tile] = touched_word;
  }
}

int chunk_for(const ConvParams& p) { return (p.gi.c % 32 == 0 && p.stride == 1) ? 32 : 16; }

template <int CHUNK, int NW>
void launch_variant(const ConvParams& p, hipStream_t s) {
  const int P = 7 * p.stride + p.k;
  size_t lds = (size_t)P * P * (CHUNK + 4) * sizeof(float);
  if (lds < 4 * 32 * 64 * sizeof(float)) lds = 4 * 32 * 64 * sizeof(float);  // partial sums reuse it
  dim3 grid(p.go.tiles(), p.go.c / 32);
  hipLaunchKernelGGL((conv_mfma_f32_kernel<CHUNK, NW>), grid, dim3(NW * 64), lds, s, p);
}

}  // namespace

bool conv_mfma_f32_supported(const ConvParams& p) {
  return p.gi.c % 16 == 0 && p.go.c % 32 == 0 && p.c_out_pad == p.go.c &&
         (long long)p.gi.h * p.gi.w * p.gi.c * 4 < (1ll << 31);  // byte offsets of the gather fit 31 bits
}

void launch_conv_mfma_f32(const ConvParams& p, hipStream_t s) {
  const int chunk = chunk_for(p);
  // low-resolution layers have few workgroups: give each one 8 waves to split K further
  const bool wide = (long long)p.go.tiles() * (p.go.c / 32) < 512;
  if (chunk == 32) {
    if (wide) launch_variant<32, 8>(p, s); else launch_variant<32, 4>(p, s);
  } else {
    if (wide) launch_variant<16, 8>(p, s); else launch_variant<16, 4>(p, s);
  }
}

}  // namespace evk
