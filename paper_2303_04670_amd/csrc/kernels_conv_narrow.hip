// Sparse incremental convolution for narrow inputs, on the matrix cores.
//
// For layers whose whole contraction K = taps x c_in is at most 128 and whose c_out is at least 16
// (the last block of 32 output channels is zero-padded): the first convolution on the event tensor
// (c_in = 2..8 channels).  With so few input channels a per-tap channel contraction is too thin
// for an MFMA, so the contraction runs over the flattened index k = tap * c_in + ci (im2col by
// addressing, nothing is materialised):
//   A[m][k] = patch[site(m) + tap offset(k)][ci(k)]   one ds_read_b32 at a per-lane offset that is
//             worked out once per workgroup and kept in registers (one register per MFMA step)
//   B[k][n] = the weights, re-laid on the host so that a lane's values for all steps are
//             contiguous; a wave keeps its whole share in registers while it walks tiles
// v_mfma_f32_16x16x4_f32, fp32 operands and accumulation (bf16-declared weights are widened, which
// is at least as accurate as the bf16 path).
//
// Workgroup = 4 waves = one 8 x 8 output tile x 32 output channels; wave = a half tile (four
// rows, 32 sites) x 16 channels as two 16 x 16 accumulator blocks that share the weight operand:
// no partial sums, and the epilogue goes straight from the accumulator registers to memory.
// Workgroups walk tiles with the grid's stride.
//
// A tile is one chain of dependent memory round trips, so they are made as few as possible: the
// occupancy words and the whole halo patch are requested together at the start (the patch
// unconditionally: it is a few KB; inactive and out-of-image sites are zeroed from the masks on
// the way into LDS), old z values and - once per workgroup - the weights as soon as the tile is
// known to be touched.  Masks, z read-modify-write, activation increment (Eq.12-14) and
// occupancy words as in the other convolution kernels.
#include <algorithm>

#include "evconv_kernels.h"

namespace evk {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kMaxK = 128;             // largest contraction length
constexpr int kMaxSteps = kMaxK / 4;   // MFMA steps of four k each
constexpr int kMaxPatchPerThread = 10; // patch elements per thread (256 threads)

__device__ __forceinline__ float act_n(int act, float v) {
  if (act == kActRelu) return fmaxf(v, 0.0f);
  if (act == kActSigmoid) return 1.0f / (1.0f + expf(-v));
  if (act == kActTanh) return tanhf(v);
  if (act == kActOneMinus) return 1.0f - v;
  return v;
}

template <int MAXE>  // patch elements per thread
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(MAXE <= 3 ? 4 : 3))) void conv_narrow_kernel(ConvParams p) {
  const size_t so = (size_t)blockIdx.z * p.st.stride;  // this workgroup's stream
  constexpr int NT = 256;
  extern __shared__ __align__(16) float s_patch[];
  __shared__ uint64_t s_occ[16];
  __shared__ unsigned s_rows[24];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = wave & 1, cb = wave >> 1;  // this wave: tile rows 4 * half .. + 3, output channels 16 * cb .. + 15
  const int kq = lane >> 4, n16 = lane & 15;               // MFMA operand lane: k = 4 * step + kq; row / column n16
  const int s = p.stride, K = p.k;
  const int H = p.gi.h, W = p.gi.w, Cin = p.gi.c, Cout = p.go.c;
  const int P = 7 * s + K;  // patch edge, <= 21
  const int CS = Cin | 1;   // odd LDS site stride
  const int k_tot = K * K * Cin, n_steps = (k_tot + 3) >> 2;
  const int cin_magic = (65536 + Cin - 1) / Cin;  // e / Cin == (e * cin_magic) >> 16 for e < 3600 (Cin <= 8)
  const int p_magic = (65536 + P - 1) / P;        // site / P likewise for site < 441
  const int k_magic = (65536 + K - 1) / K;        // tap / K likewise for tap < 49
  __shared__ int s_koff[kMaxK];

  // once per workgroup: per step the LDS position of the patch element this lane multiplies for
  // its site of the first row block (the second block's lies `blk1` further on).  Beyond taps x
  // c_in it is the position of a zero kept behind the patch: the operand is then an explicit
  // zero, not a patch element times a zero weight (the element may be infinite or NaN).
  const int zero_at = P * P * CS;
  const int blk1 = 2 * s * P * CS;
  const int site0 = ((4 * half + (n16 >> 3)) * s * P + (n16 & 7) * s) * CS;
  if (tid == 0) s_patch[zero_at] = s_patch[zero_at + blk1] = 0.0f;  // (never overwritten: the patch ends before them)
  // per patch element of this thread: where it goes in LDS, its bit in the row masks and its
  // offset in the input relative to the patch origin (the same for every tile)
  int e_lds[MAXE], e_bit[MAXE], e_goff[MAXE];
  const int total = P * P * Cin;
#pragma unroll
  for (int j = 0; j < MAXE; ++j) {
    const int e = tid + j * NT;
    e_lds[j] = -1; e_bit[j] = 0; e_goff[j] = 0;
    if (e < total) {
      const int site = (e * cin_magic) >> 16, c = e - site * Cin;
      const int py = (site * p_magic) >> 16, px = site - py * P;
      e_lds[j] = site * CS + c;
      e_bit[j] = py * 32 + px;
      e_goff[j] = ((py * W + px) * Cin + c) * 4;
    }
  }
  // the weights of this wave's lane, one per step, fetched when the first touched tile is met
  // (a workgroup without one leaves without reading them)
  float wreg[kMaxSteps];
  bool staged = false;
  const int co = blockIdx.y * 32 + cb * 16 + n16;

  for (int tile = blockIdx.x; tile < p.go.tiles(); tile += gridDim.x) {
    const int tile_y = tile / p.go.tx, tile_x = tile - tile_y * p.go.tx;
    const int iy0 = tile_y * 8 * s - p.pad, ix0 = tile_x * 8 * s - p.pad;
    const int rty0 = iy0 >> 3, rtx0 = ix0 >> 3;
    const int rny = ((iy0 + P - 1) >> 3) - rty0 + 1, rnx = ((ix0 + P - 1) >> 3) - rtx0 + 1;
    // requests first: the occupancy words under the halo and every element of the patch
    uint64_t occ_w = 0;
    if (tid < 16) {
      const int ry = tid >> 2, rx = tid & 3;
      const int ty = rty0 + ry, tx = rtx0 + rx;
      if (ry < rny && rx < rnx && ty >= 0 && ty < p.gi.ty && tx >= 0 && tx < p.gi.tx)
        occ_w = p.dense ? ~0ull : at_stream(p.occ_in, so)[ty * p.gi.tx + tx];
    }
    const __amdgpu_buffer_rsrc_t in_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)at_stream(p.in, so), 0, H * W * Cin * 4, 0x00020000);
    // (rows outside the image give an out-of-range offset: the load returns 0; columns outside it
    // read a neighbouring row's site, which the mask below discards; a thread without a j-th
    // element gets an out-of-range offset as well)
    const int origin = (iy0 * W + ix0) * Cin * 4;
    float pre[MAXE];
#pragma unroll
    for (int j = 0; j < MAXE; ++j) {
      const unsigned off = e_lds[j] >= 0 ? (unsigned)(origin + e_goff[j]) : 0x80000000u;
      pre[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(in_rsrc, off, 0, 0));
    }
    __syncthreads();  // the previous tile's masks and patch are no longer in use
    if (tid < 16) s_occ[tid] = occ_w;
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

    // accumulator element (block r, register i, lane) = local site 16 * r + 4 * kq + i of the half
    // tile, channel n16 of this wave's 16
    float z_old[2][4];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ls = 16 * r + 4 * kq + i;
        z_old[r][i] = 0.0f;
        if (!p.dense && co < Cout && ((my_touched >> ls) & 1u)) {
          const int oy = tile_y * 8 + 4 * half + (ls >> 3), ox = tile_x * 8 + (ls & 7);
          z_old[r][i] = at_stream(p.z, so)[((size_t)oy * p.go.w + ox) * Cout + co];
        }
      }
    if (!staged) {
      // k -> LDS position of the patch element it multiplies, relative to the output site's patch
      // origin; beyond taps x c_in the position of the zero behind the patch, relative likewise
      if (tid < kMaxK) {
        const int k = tid;
        int off = zero_at;
        if (k < k_tot) {
          const int tap = (k * cin_magic) >> 16, ci = k - tap * Cin;
          const int ky = (tap * k_magic) >> 16, kx = tap - ky * K;
          off = (ky * P + kx) * CS + ci;
        }
        s_koff[k] = off;
      }
      // re-laid weights: [32-channel group][block of 16][lane][step]: a lane's share is 128 bytes
      const float4* wsrc = (const float4*)((const float*)p.w + (((size_t)blockIdx.y * 2 + cb) * 64 + lane) * kMaxSteps);
#pragma unroll
      for (int v = 0; v < kMaxSteps / 4; ++v) {
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if (4 * v < n_steps) t = wsrc[v];
        wreg[4 * v] = t.x; wreg[4 * v + 1] = t.y; wreg[4 * v + 2] = t.z; wreg[4 * v + 3] = t.w;
      }
      staged = true;
    }
    // patch into LDS: inactive and out-of-image sites become zeros
#pragma unroll
    for (int j = 0; j < MAXE; ++j)
      if (e_lds[j] >= 0) s_patch[e_lds[j]] = ((s_rows[e_bit[j] >> 5] >> (e_bit[j] & 31)) & 1u) ? pre[j] : 0.0f;
    __syncthreads();
    if (my_touched == 0) continue;  // (uniform per wave; the barriers of the next tile are met by all waves)

    floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    {
      // the two row blocks of the half tile: rows 4 * half + (n16 >> 3) and two rows further down
      // (the distance is re-materialised per tile so that the second block's 32 addresses are
      // formed at their use instead of living in registers across the tile loop)
      int blk1_v = blk1, site0_v = site0;
      asm volatile("" : "+v"(blk1_v), "+v"(site0_v));
      // in batches of eight steps: the operand reads of a batch, then its matrix instructions
#pragma unroll
      for (int s0 = 0; s0 < kMaxSteps; s0 += 8) {
        if (s0 >= n_steps) break;
        int ko[8];
        float a0[8], a1[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) ko[j] = s_koff[4 * (s0 + j) + kq];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          // (the zero behind the patch is addressed absolutely: site0 is taken off again)
          const int at = ko[j] >= zero_at ? ko[j] : ko[j] + site0_v;
          a0[j] = s_patch[at];
          a1[j] = s_patch[at + blk1_v];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a0[j], wreg[s0 + j], acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[j], wreg[s0 + j], acc1, 0, 0, 0);
        }
      }
    }

    // epilogue straight from the accumulator registers
    unsigned nz = 0;  // nonzero output sites of this wave (bits of its 32-site half)
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ls = 16 * r + 4 * kq + i;
        const int oy = tile_y * 8 + 4 * half + (ls >> 3), ox = tile_x * 8 + (ls & 7);
        const bool on = ((my_touched >> ls) & 1u) && co < Cout;  // (c_out rounded up to 32: surplus lanes own nothing)
        float o = 0.0f;
        if (on) {
          const size_t e = ((size_t)oy * p.go.w + ox) * Cout + co;
          const float v = r == 0 ? acc0[i] : acc1[i];
          if (p.dense) {
            const float z = v + (p.bias ? p.bias[co] : 0.0f);
            at_stream(p.z, so)[e] = z;
            o = act_n(p.act, z);
          } else {
            const float z_new = z_old[r][i] + v;
            at_stream(p.z, so)[e] = z_new;
            o = (p.act == kActNone) ? v : act_n(p.act, z_new) - act_n(p.act, z_old[r][i]);
          }
          at_stream(p.out, so)[e] = o;
        }
        const uint64_t bal = __ballot(on && o != 0.0f);  // 16 lanes (channels) per site: sites 16 * r + 4 * g + i
#pragma unroll
        for (int g = 0; g < 4; ++g)
          if ((bal >> (16 * g)) & 0xffffull) nz |= 1u << (16 * r + 4 * g + i);
      }
    if (lane == 0) {
      const uint64_t mine = (uint64_t)(p.dense ? my_touched : nz) << (32 * half);
      if (mine) atomicOr((unsigned long long*)&at_stream(p.occ_out, so)[tile], (unsigned long long)mine);  // pre-zeroed word
      if (blockIdx.y == 0 && cb == 0) {
        const uint64_t t = (uint64_t)my_touched << (32 * half);
        if (t) atomicOr((unsigned long long*)&at_stream(p.occ_touched, so)[tile], (unsigned long long)t);
      }
    }
  }  // tiles
}

}  // namespace

bool conv_narrow_supported(const ConvParams& p) {
  const int k_tot = p.k * p.k * p.gi.c;
  const int P = 7 * p.stride + p.k;
  return k_tot <= kMaxK && p.gi.c <= 8 && p.go.c >= 16 && p.c_out_pad == (p.go.c + 31) / 32 * 32 && p.n_fused == 0 &&
         P * P * p.gi.c <= kMaxPatchPerThread * 256 &&
         (long long)p.gi.h * p.gi.w * p.gi.c * 4 < (1ll << 31);  // byte offsets of the gather fit 31 bits
}

// re-laid weights: floats for c_out_pad output channels, and the position of W[k][co]
// (k = tap * c_in + ci): [co / 32][(co % 32) / 16][lane = (k % 4) * 16 + co % 16][step = k / 4]
size_t conv_narrow_weight_floats(int c_out_pad) { return (size_t)(c_out_pad / 32) * 2 * 64 * kMaxSteps; }
size_t conv_narrow_weight_index(int k, int co) {
  return ((size_t)((co >> 5) * 2 + ((co & 31) >> 4)) * 64 + (size_t)(k & 3) * 16 + (co & 15)) * kMaxSteps + (k >> 2);
}

void launch_conv_narrow(const ConvParams& p, hipStream_t s) {
  const int P = 7 * p.stride + p.k;
  const int cs = p.gi.c | 1;
  // the patch, then room for the two zeros that stand in for operands beyond taps x c_in
  const size_t lds = ((size_t)P * P * cs + 2 * p.stride * P * cs + 1) * sizeof(float);
  // workgroups walk the tiles with the grid's stride; enough of them to fill the chip's resident
  // slots (a tile is one chain of dependent memory round trips, so few long walks are slow)
  dim3 grid(std::min(p.go.tiles(), std::max(4096 / p.st.n, 256)), p.c_out_pad / 32, p.st.n);
  if (P * P * p.gi.c <= 3 * 256) hipLaunchKernelGGL(conv_narrow_kernel<3>, grid, dim3(256), lds, s, p);
  else hipLaunchKernelGGL(conv_narrow_kernel<kMaxPatchPerThread>, grid, dim3(256), lds, s, p);
}

}  // namespace evk
