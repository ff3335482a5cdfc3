// gfx950 kernels: increment builder, elementwise / structural increment operators, global
// average pool, output integration, ordered list compaction.
//
// Conventions: tensors are H x W x C fp32; a tile is 8 x 8 sites and its occupancy word has
// bit (y%8)*8 + x%8 set for an active site; tiles are row-major.  Nothing here uses
// floating-point atomics: every accumulated element has exactly one writer, so results are
// run-to-run bit-reproducible.
#include "evconv_kernels.h"

namespace evk {

namespace {

__device__ __forceinline__ bool occ_bit(const uint64_t* __restrict__ occ, int tx, int y, int x) {
  uint64_t w = occ[(y >> 3) * tx + (x >> 3)];
  return (w >> (((y & 7) << 3) | (x & 7))) & 1ull;
}

__device__ __forceinline__ float apply_act(int act, float v) {
  if (act == kActRelu) return fmaxf(v, 0.0f);
  if (act == kActSigmoid) return 1.0f / (1.0f + expf(-v));
  if (act == kActTanh) return tanhf(v);
  if (act == kActOneMinus) return 1.0f - v;
  return v;
}

// in-bounds mask of tile (tile_y, tile_x) of an h x w grid, bit layout as the occupancy words
__device__ __forceinline__ uint64_t inbounds_word(int h, int w, int tile_y, int tile_x) {
  int rows = min(8, h - tile_y * 8), cols = min(8, w - tile_x * 8);
  uint64_t row = (cols >= 8) ? 0xffull : ((1ull << cols) - 1);
  uint64_t m = 0;
  for (int r = 0; r < rows; ++r) m |= row << (8 * r);
  return m;
}

}  // namespace

// =============================================================================== builder
// One workgroup = 8 wavefronts = an 8-row x 64-column strip (8 tiles).  Wave r reads row r with
// 256-byte coalesced loads per channel; its ballot is the 64-column activity of that row.  The
// eight ballots are transposed through LDS into eight tile occupancy words.
__global__ __launch_bounds__(512) void builder_kernel(BuilderParams p) {
  {
    const size_t so = (size_t)blockIdx.z * p.st.stride;
    p.in = at_stream(p.in, (size_t)blockIdx.z * p.in_stride);
    p.x_prev = at_stream(p.x_prev, so); p.dx = at_stream(p.dx, so);
    p.occ = at_stream(p.occ, so); p.clear = at_stream(p.clear, so);
  }
  __shared__ uint64_t s_rows[8];
  const int lane = threadIdx.x & 63;
  const int r = threadIdx.x >> 6;
  const int y = blockIdx.y * 8 + r;
  const int x = blockIdx.x * 64 + lane;
  const int hw = p.g.h * p.g.w;
  const bool inb = (y < p.g.h) && (x < p.g.w);
  bool any = false;
  if (inb) {
    const int site = y * p.g.w + x;
    for (int c = 0; c < p.g.c; ++c) {
      const int e = c * hw + site;
      float d;
      if (p.mode == kBuildFrame) {
        const float xt = p.in[e];
        d = xt - p.x_prev[e];          // Eq.1: one binary32 subtraction
        p.x_prev[e] = xt;
      } else if (p.mode == kBuildIncrement) {
        d = p.in[e];
        p.x_prev[e] = p.x_prev[e] + d;
      } else if (p.mode == kBuildIncrementDense) {
        d = p.x_prev[e] + p.in[e];     // dense recompute of a supplied increment: emit x(n)
        p.x_prev[e] = d;
      } else {
        d = p.in[e];
        p.x_prev[e] = d;
      }
      p.dx[(size_t)site * p.g.c + c] = d;
      any |= (d != 0.0f);
    }
  }
  const uint64_t row_mask = __ballot(any);
  if (lane == 0) s_rows[r] = row_mask;
  __syncthreads();
  if (threadIdx.x < 8) {
    const int j = threadIdx.x;
    const int tile_x = blockIdx.x * 8 + j;
    if (tile_x < p.g.tx) {
      uint64_t word = 0;
      for (int rr = 0; rr < 8; ++rr) word |= ((s_rows[rr] >> (8 * j)) & 0xffull) << (8 * rr);
      if (p.mode >= kBuildReset) word = 0;
      p.occ[blockIdx.y * p.g.tx + tile_x] = word;
    }
  }
  // clear the per-node occupancy words that the layer kernels OR into
  if (p.clear) {
    const int nthreads = gridDim.x * gridDim.y * blockDim.x;
    const int gtid = (blockIdx.y * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x;
    for (int i = gtid; i < p.n_clear; i += nthreads) p.clear[i] = 0;
  }
}

void launch_builder(const BuilderParams& p, hipStream_t s) {
  dim3 grid((p.g.w + 63) / 64, (p.g.h + 7) / 8, p.st.n);
  hipLaunchKernelGGL(builder_kernel, grid, dim3(512), 0, s, p);
}

// =============================================================================== elementwise
// One workgroup per output tile.  Wave 0 derives the tile's touched word and the list of
// touched sites; then the 256 threads walk (touched site, channel vector) pairs with the
// channel index fastest, so global accesses are contiguous runs of C floats per site.
constexpr int kEwVecPerBlock = 16;  // channel vectors per workgroup: wide layers split over blockIdx.y

template <int VEC> struct VecT { float v[VEC]; };
template <int VEC> __device__ __forceinline__ VecT<VEC> ldv(const float* ptr) {
  VecT<VEC> r;
  if (VEC == 4) {
    const float4 t = *(const float4*)ptr;  // channel counts are multiples of 4 and buffers 256-byte aligned
    r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
  } else {
#pragma unroll
    for (int i = 0; i < VEC; ++i) r.v[i] = ptr[i];
  }
  return r;
}
template <int VEC> __device__ __forceinline__ void stv(float* ptr, const VecT<VEC>& x) {
  if (VEC == 4) {
    *(float4*)ptr = make_float4(x.v[0], x.v[1], x.v[2], x.v[3]);
  } else {
#pragma unroll
    for (int i = 0; i < VEC; ++i) ptr[i] = x.v[i];
  }
}
template <int VEC> __device__ __forceinline__ VecT<VEC> zerov() {
  VecT<VEC> r;
#pragma unroll
  for (int i = 0; i < VEC; ++i) r.v[i] = 0.0f;
  return r;
}

template <int VEC>
__global__ __launch_bounds__(256) void elementwise_kernel(EwParams p) {
  {
    const size_t so = (size_t)blockIdx.z * p.st.stride;
    p.a = at_stream(p.a, so); p.occ_a = at_stream(p.occ_a, so);
    p.b = at_stream(p.b, so); p.occ_b = at_stream(p.occ_b, so);
    p.z = at_stream(p.z, so); p.z2 = at_stream(p.z2, so); p.out = at_stream(p.out, so);
    p.occ_out = at_stream(p.occ_out, so); p.occ_touched = at_stream(p.occ_touched, so);
    p.step = at_stream(p.step, so);
  }
  __shared__ int s_sites[64];
  __shared__ unsigned char s_src[64];  // upsample: which of the four source sites are active
  __shared__ unsigned s_flags[2];
  __shared__ uint64_t s_word, s_wa, s_wb;
  const int tid = threadIdx.x;
  const int tile = blockIdx.x;
  const int tile_y = tile / p.go.tx, tile_x = tile - tile_y * p.go.tx;

  if (tid < 64) {
    const int ly = tid >> 3, lx = tid & 7;
    const int oy = tile_y * 8 + ly, ox = tile_x * 8 + lx;
    const bool inb = oy < p.go.h && ox < p.go.w;
    bool t = false;
    uint64_t wa = 0, wb = 0;
    unsigned src = 15;
    if (p.dense) {
      t = inb;
      wa = wb = ~0ull;
    } else if (p.op == kEwAdd || p.op == kEwConcat || p.op == kEwMul) {
      wa = p.occ_a[tile];
      wb = p.occ_b[tile];
      t = ((wa | wb) >> tid) & 1ull;
    } else if (p.op == kEwAct || p.op == kEwPoolAcc || p.op == kEwSparsify) {
      wa = p.occ_a[tile];
      t = (wa >> tid) & 1ull;
    } else if (p.op == kEwUp2x || p.op == kEwConcatUp) {
      src = 0;
      if (p.op == kEwConcatUp) wb = p.occ_b[tile];
      if (inb) {
        const int iy = oy >> 1, ix = ox >> 1;
        const int y0 = (oy & 1) ? iy : max(iy - 1, 0), y1 = (oy & 1) ? min(iy + 1, p.ga.h - 1) : iy;
        const int x0 = (ox & 1) ? ix : max(ix - 1, 0), x1 = (ox & 1) ? min(ix + 1, p.ga.w - 1) : ix;
        src = (unsigned)occ_bit(p.occ_a, p.ga.tx, y0, x0) | ((unsigned)occ_bit(p.occ_a, p.ga.tx, y0, x1) << 1) |
              ((unsigned)occ_bit(p.occ_a, p.ga.tx, y1, x0) << 2) | ((unsigned)occ_bit(p.occ_a, p.ga.tx, y1, x1) << 3);
        t = src != 0 || (p.op == kEwConcatUp && ((wb >> tid) & 1ull));
      }
    } else {  // kEwPoolMax: windows that contain an active input site
      if (inb) {
        for (int ky = 0; ky < p.k; ++ky) {
          const int iy = oy * p.stride - p.pad + ky;
          if ((unsigned)iy >= (unsigned)p.ga.h) continue;
          for (int kx = 0; kx < p.k; ++kx) {
            const int ix = ox * p.stride - p.pad + kx;
            if ((unsigned)ix >= (unsigned)p.ga.w) continue;
            t |= occ_bit(p.occ_a, p.ga.tx, iy, ix);
          }
        }
      }
    }
    s_src[tid] = (unsigned char)src;
    const uint64_t word = __ballot(t);
    if (t) s_sites[__popcll(word & ((1ull << tid) - 1))] = tid;
    if (tid == 0) { s_word = word; s_wa = wa; s_wb = wb; s_flags[0] = 0; s_flags[1] = 0; }
  }
  __syncthreads();
  const uint64_t word = s_word;
  if (word == 0) return;
  const uint64_t wa = s_wa, wb = s_wb;
  const int n_sites = __popcll(word);
  const int C = p.go.c;
  // channel vectors [v0, v0 + cv) of every touched site belong to this workgroup
  const int cv_all = C / VEC;
  const int v0 = blockIdx.y * kEwVecPerBlock;
  const int cv = min(kEwVecPerBlock, cv_all - v0);
  const int total = n_sites * cv;

  // sites at which this thread produced a nonzero element; the waves' ORs meet in LDS afterwards
  // (one LDS atomic per element would be served lane by lane where the lanes share a site)
  uint64_t nz_sites = 0;
  for (int e = tid; e < total; e += 256) {
    const int r = e / cv, v = v0 + (e - r * cv);
    const int site = s_sites[r];
    const int oy = tile_y * 8 + (site >> 3), ox = tile_x * 8 + (site & 7);
    const size_t q = (size_t)oy * p.go.w + ox;
    const int c = v * VEC;
    VecT<VEC> lin, lin_b;
    if (p.op == kEwMul) {  // the two factors' increments (full values in a regular forward pass)
      const bool on_a = (wa >> site) & 1ull, on_b = (wb >> site) & 1ull;
      lin = on_a ? ldv<VEC>(&p.a[q * C + c]) : zerov<VEC>();
      lin_b = on_b ? ldv<VEC>(&p.b[q * C + c]) : zerov<VEC>();
    } else if (p.op == kEwAdd) {
      const bool on_a = (wa >> site) & 1ull, on_b = (wb >> site) & 1ull;
      const VecT<VEC> va = on_a ? ldv<VEC>(&p.a[q * C + c]) : zerov<VEC>();
      const VecT<VEC> vb = on_b ? ldv<VEC>(&p.b[q * C + c]) : zerov<VEC>();
#pragma unroll
      for (int i = 0; i < VEC; ++i) lin.v[i] = va.v[i] + vb.v[i];
    } else if (p.op == kEwAct || p.op == kEwPoolAcc || p.op == kEwSparsify) {
      lin = ldv<VEC>(&p.a[q * C + c]);
    } else if (p.op == kEwConcat) {
      const bool on_a = (wa >> site) & 1ull, on_b = (wb >> site) & 1ull;
      const int ca = p.ga.c, cb = p.gb.c;
      if (VEC == 4) {  // c_a % 4 == 0: a vector never straddles the two inputs
        lin = c < ca ? (on_a ? ldv<VEC>(&p.a[q * ca + c]) : zerov<VEC>())
                     : (on_b ? ldv<VEC>(&p.b[q * cb + c - ca]) : zerov<VEC>());
      } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          const int cc = c + i;
          lin.v[i] = cc < ca ? (on_a ? p.a[q * ca + cc] : 0.0f) : (on_b ? p.b[q * cb + cc - ca] : 0.0f);
        }
      }
    } else if (p.op == kEwUp2x || (p.op == kEwConcatUp && c < p.ga.c)) {
      // (kEwConcatUp runs with whole vectors only: c_a % 4 == 0, so a vector is on one side)
      const int CA = p.ga.c;  // channels of the stored tensor (== C for a bare up-sampling)
      const int iy = oy >> 1, ix = ox >> 1;
      const int y0 = (oy & 1) ? iy : max(iy - 1, 0), y1 = (oy & 1) ? min(iy + 1, p.ga.h - 1) : iy;
      const int x0 = (ox & 1) ? ix : max(ix - 1, 0), x1 = (ox & 1) ? min(ix + 1, p.ga.w - 1) : ix;
      const float wy0 = (oy & 1) ? 0.75f : 0.25f, wy1 = 1.0f - wy0;
      const float wx0 = (ox & 1) ? 0.75f : 0.25f, wx1 = 1.0f - wx0;
      const unsigned src = s_src[site];
      const VecT<VEC> v00 = (src & 1) ? ldv<VEC>(&p.a[((size_t)y0 * p.ga.w + x0) * CA + c]) : zerov<VEC>();
      const VecT<VEC> v01 = (src & 2) ? ldv<VEC>(&p.a[((size_t)y0 * p.ga.w + x1) * CA + c]) : zerov<VEC>();
      const VecT<VEC> v10 = (src & 4) ? ldv<VEC>(&p.a[((size_t)y1 * p.ga.w + x0) * CA + c]) : zerov<VEC>();
      const VecT<VEC> v11 = (src & 8) ? ldv<VEC>(&p.a[((size_t)y1 * p.ga.w + x1) * CA + c]) : zerov<VEC>();
#pragma unroll
      for (int i = 0; i < VEC; ++i)
        lin.v[i] = wy0 * (wx0 * v00.v[i] + wx1 * v01.v[i]) + wy1 * (wx0 * v10.v[i] + wx1 * v11.v[i]);
    } else if (p.op == kEwConcatUp) {  // the second operand's channels
      const bool on_b = (wb >> site) & 1ull;
      lin = on_b ? ldv<VEC>(&p.b[q * p.gb.c + c - p.ga.c]) : zerov<VEC>();
    } else {  // kEwPoolMax: p.a is the accumulated pool input, p.z the cached window maximum
#pragma unroll
      for (int i = 0; i < VEC; ++i) lin.v[i] = -INFINITY;
      if (p.k == 3) {
        // the usual window: nine loads requested together (an out-of-image tap reads the window's
        // centre instead and is left out of the maximum), then the maxima in the same order
        VecT<VEC> t[9];
        bool ok[9];
        const int cy = min(max(oy * p.stride - p.pad + 1, 0), p.ga.h - 1), cx = min(max(ox * p.stride - p.pad + 1, 0), p.ga.w - 1);
#pragma unroll
        for (int j = 0; j < 9; ++j) {
          const int iy = oy * p.stride - p.pad + j / 3, ix = ox * p.stride - p.pad + j % 3;
          ok[j] = (unsigned)iy < (unsigned)p.ga.h && (unsigned)ix < (unsigned)p.ga.w;
          t[j] = ldv<VEC>(&p.a[((size_t)(ok[j] ? iy : cy) * p.ga.w + (ok[j] ? ix : cx)) * C + c]);
        }
#pragma unroll
        for (int j = 0; j < 9; ++j)
#pragma unroll
          for (int i = 0; i < VEC; ++i) lin.v[i] = ok[j] ? fmaxf(lin.v[i], t[j].v[i]) : lin.v[i];
      } else
      for (int ky = 0; ky < p.k; ++ky) {
        const int iy = oy * p.stride - p.pad + ky;
        if ((unsigned)iy >= (unsigned)p.ga.h) continue;
        for (int kx = 0; kx < p.k; ++kx) {
          const int ix = ox * p.stride - p.pad + kx;
          if ((unsigned)ix >= (unsigned)p.ga.w) continue;
          const VecT<VEC> t = ldv<VEC>(&p.a[((size_t)iy * p.ga.w + ix) * C + c]);
#pragma unroll
          for (int i = 0; i < VEC; ++i) lin.v[i] = fmaxf(lin.v[i], t.v[i]);
        }
      }
    }

    float* zq = p.z ? &p.z[q * C + c] : nullptr;
    if (p.op == kEwPoolAcc) {
      VecT<VEC> acc = lin;
      if (!p.dense) {
        const VecT<VEC> old = ldv<VEC>(zq);
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc.v[i] = old.v[i] + lin.v[i];
      }
      stv<VEC>(zq, acc);
      continue;
    }
    VecT<VEC> o;
    bool nz = false;
    if (p.op == kEwMul) {
      // Eq.15-17: y_inc = (x1acc + x1_inc) * x2_inc + x2acc * x1_inc, then both accumulators
      // advance.  Explicitly rounded operations: no fused multiply-add, so the result is the
      // same single-rounded sequence on any implementation.
      float* z2q = &p.z2[q * C + c];
      if (p.dense) {
        stv<VEC>(zq, lin);
        stv<VEC>(z2q, lin_b);
#pragma unroll
        for (int i = 0; i < VEC; ++i) o.v[i] = lin.v[i] * lin_b.v[i];
      } else {
#pragma clang fp contract(off)
        const VecT<VEC> a1 = ldv<VEC>(zq), a2 = ldv<VEC>(z2q);
        VecT<VEC> n1, n2;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          n1.v[i] = a1.v[i] + lin.v[i];
          n2.v[i] = a2.v[i] + lin_b.v[i];
          const float t1 = n1.v[i] * lin_b.v[i], t2 = a2.v[i] * lin.v[i];
          o.v[i] = t1 + t2;
        }
        stv<VEC>(zq, n1);
        stv<VEC>(z2q, n2);
      }
    } else if (p.op == kEwSparsify) {
      // Eq.3-8: x_corr = delta + x_inc; y_inc = k floor(0.5 + x_corr / k); delta = x_corr - y_inc
      const float k = p.dense ? 0.0f : *p.step;
      VecT<VEC> d_new = zerov<VEC>();
      o = lin;
      if (k > 0.0f) {
#pragma clang fp contract(off)  // the residual is x_corr minus the rounded product, not a fused form
        const VecT<VEC> d_old = ldv<VEC>(zq);
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          // (an element with a zero increment emits nothing and keeps its residual: |delta| <= k/2)
          const float x_corr = d_old.v[i] + lin.v[i];
          const bool moved = lin.v[i] != 0.0f;
          o.v[i] = moved ? k * floorf(0.5f + x_corr / k) : 0.0f;
          d_new.v[i] = moved ? x_corr - o.v[i] : d_old.v[i];
        }
      }
      if (p.dense || k > 0.0f) stv<VEC>(zq, d_new);  // a refresh clears the residual
    } else if (p.op == kEwPoolMax) {
      const VecT<VEC> m_old = ldv<VEC>(zq);
      stv<VEC>(zq, lin);
#pragma unroll
      for (int i = 0; i < VEC; ++i) o.v[i] = p.dense ? lin.v[i] : lin.v[i] - m_old.v[i];
    } else if (p.keeps_z) {
      if (p.dense) {
        stv<VEC>(zq, lin);
#pragma unroll
        for (int i = 0; i < VEC; ++i) o.v[i] = apply_act(p.act, lin.v[i]);
      } else {
        const VecT<VEC> z_old = ldv<VEC>(zq);
        VecT<VEC> z_new;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          z_new.v[i] = z_old.v[i] + lin.v[i];
          o.v[i] = (p.act == kActNone) ? lin.v[i] : apply_act(p.act, z_new.v[i]) - apply_act(p.act, z_old.v[i]);
        }
        stv<VEC>(zq, z_new);
      }
    } else {
      o = lin;
    }
    stv<VEC>(&p.out[q * C + c], o);
#pragma unroll
    for (int i = 0; i < VEC; ++i) nz |= (o.v[i] != 0.0f);
    if (nz) nz_sites |= 1ull << site;
  }
  if (p.op == kEwPoolAcc) return;
  if (!p.structural) {
    unsigned lo = (unsigned)nz_sites, hi = (unsigned)(nz_sites >> 32);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
      lo |= __shfl_xor(lo, m);
      hi |= __shfl_xor(hi, m);
    }
    if ((tid & 63) == 0) {
      if (lo) atomicOr(&s_flags[0], lo);
      if (hi) atomicOr(&s_flags[1], hi);
    }
  }
  __syncthreads();
  if (tid == 0) {
    const uint64_t flags = (uint64_t)s_flags[0] | ((uint64_t)s_flags[1] << 32);
    if (p.structural || p.dense) {
      if (blockIdx.y == 0) p.occ_out[tile] = word;
    } else if (flags) {
      atomicOr((unsigned long long*)&p.occ_out[tile], (unsigned long long)flags);  // pre-zeroed word
    }
    if (blockIdx.y == 0) p.occ_touched[tile] = word;
  }
}

void launch_elementwise(const EwParams& p, hipStream_t s) {
  bool vec4 = (p.go.c % 4) == 0;
  if (p.op == kEwConcat || p.op == kEwConcatUp) vec4 = vec4 && (p.ga.c % 4) == 0;
  const int cv_all = p.go.c / (vec4 ? 4 : 1);
  dim3 grid(p.go.tiles(), (cv_all + kEwVecPerBlock - 1) / kEwVecPerBlock, p.st.n);
  if (vec4) hipLaunchKernelGGL(elementwise_kernel<4>, grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL(elementwise_kernel<1>, grid, dim3(256), 0, s, p);
}

// =============================================================================== global avg pool
// Workgroup = 64 channels x 4 row slices: slice s sums the active sites of tile rows s and s + 4
// of every tile, a row's eight loads in flight together; the four partial sums are added in a
// fixed order.  Sites are visited in a fixed order throughout, so the fp32 sum is reproducible.
__global__ __launch_bounds__(256) void gap_kernel(GapParams p) {
  {
    const size_t so = (size_t)blockIdx.z * p.st.stride;
    p.a = at_stream(p.a, so); p.occ_a = at_stream(p.occ_a, so); p.z = at_stream(p.z, so);
    p.out = at_stream(p.out, so); p.occ_out = at_stream(p.occ_out, so); p.occ_touched = at_stream(p.occ_touched, so);
  }
  __shared__ float s_part[4][64];
  const int cl = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  const int C = p.ga.c;
  const bool c_ok = c < C;
  bool any = false;
  float sum = 0.0f;
  for (int t = 0; t < p.ga.tiles(); ++t) {
    const int tile_y = t / p.ga.tx, tile_x = t - tile_y * p.ga.tx;
    const uint64_t w = p.dense ? inbounds_word(p.ga.h, p.ga.w, tile_y, tile_x) : p.occ_a[t];
    any |= (w != 0);
    for (int r = slice; r < 8; r += 4) {
      const unsigned bits = (unsigned)(w >> (8 * r)) & 0xffu;
      if (bits == 0) continue;
      const int y = tile_y * 8 + r;
      float v[8];
#pragma unroll
      for (int x = 0; x < 8; ++x)
        v[x] = (((bits >> x) & 1u) && c_ok) ? p.a[((size_t)y * p.ga.w + tile_x * 8 + x) * C + c] : 0.0f;
#pragma unroll
      for (int x = 0; x < 8; ++x) sum += v[x];
    }
  }
  if (!any) return;  // (the same for every thread)
  s_part[slice][cl] = sum;
  __syncthreads();
  if (slice != 0) return;
  bool nz = false;
  if (c_ok) {
    const float lin = ((s_part[0][cl] + s_part[1][cl]) + (s_part[2][cl] + s_part[3][cl])) / (float)(p.ga.h * p.ga.w);
    float o;
    if (p.dense) {
      p.z[c] = lin;
      o = apply_act(p.act, lin);
    } else {
      const float z_old = p.z[c], z_new = z_old + lin;
      p.z[c] = z_new;
      o = (p.act == kActNone) ? lin : apply_act(p.act, z_new) - apply_act(p.act, z_old);
    }
    p.out[c] = o;
    nz = (o != 0.0f);
  }
  const bool structural = (p.act == kActNone) || p.dense;
  const uint64_t b = __ballot(nz);
  if (cl == 0) {
    if (structural) { if (c == 0) p.occ_out[0] = 1ull; }
    else if (b) atomicOr((unsigned long long*)p.occ_out, 1ull);
    if (c == 0) p.occ_touched[0] = 1ull;
  }
}

void launch_gap(const GapParams& p, hipStream_t s) {
  hipLaunchKernelGGL(gap_kernel, dim3((p.ga.c + 63) / 64, 1, p.st.n), dim3(256), 0, s, p);
}

// =============================================================================== Eq.2
__global__ __launch_bounds__(256) void integrate_kernel(IntegrateParams p) {
  {
    const size_t so = (size_t)blockIdx.z * p.st.stride;
    p.delta = at_stream(p.delta, so); p.occ = at_stream(p.occ, so);
    p.y = at_stream(p.y, so); p.dy = at_stream(p.dy, so);
  }
  const int site = blockIdx.x * 256 + threadIdx.x;
  const int hw = p.g.h * p.g.w;
  if (site >= hw) return;
  const int y = site / p.g.w, x = site - y * p.g.w;
  const bool on = p.mode != kIntStep || occ_bit(p.occ, p.g.tx, y, x);
  for (int c = 0; c < p.g.c; ++c) {
    const int e = c * hw + site;
    const float v = on ? p.delta[(size_t)site * p.g.c + c] : 0.0f;
    if (p.mode == kIntStep) {
      if (on) p.y[e] += v;
      p.dy[e] = v;
    } else if (p.mode == kIntReset) {
      p.y[e] = v;
      p.dy[e] = 0.0f;
    } else {
      p.dy[e] = v - p.y[e];
      p.y[e] = v;
    }
  }
}

void launch_integrate(const IntegrateParams& p, hipStream_t s) {
  hipLaunchKernelGGL(integrate_kernel, dim3((p.g.sites() + 255) / 256, 1, p.st.n), dim3(256), 0, s, p);
}

// =============================================================================== recurrent state
// Workgroup = one 8 x 8 tile; thread = (site, channel) pairs strided over the tile's active sites.
__global__ __launch_bounds__(256) void delay_kernel(DelayParams p) {
  const size_t so = (size_t)blockIdx.z * p.st.stride;
  const float* src = at_stream(p.src_out, so);
  float* z = at_stream(p.z, so);
  float* out = at_stream(p.out, so);
  const int tile = blockIdx.x;
  const int tile_y = tile / p.g.tx, tile_x = tile - tile_y * p.g.tx;
  const int rows = min(8, p.g.h - tile_y * 8), cols = min(8, p.g.w - tile_x * 8);
  uint64_t inb = 0;
  {
    const uint64_t rowbits = cols >= 8 ? 0xffull : ((1ull << cols) - 1ull);
    for (int r = 0; r < rows; ++r) inb |= rowbits << (8 * r);
  }
  const uint64_t saved = at_stream(p.occ_saved, so)[tile] & inb;
  // sites visited: all of the tile in or after a regular pass, the delayed node's active set otherwise
  const uint64_t word = (p.dense || p.last_dense) ? inb : saved;
  if (threadIdx.x == 0) {  // this workgroup is the tile's only writer
    at_stream(p.occ_out, so)[tile] = word;
    at_stream(p.occ_touched, so)[tile] = word;
  }
  const int C = p.g.c;
  const int n_active = __popcll(word);
  __shared__ unsigned char s_site[64];  // the visited sites in ascending order
  if (threadIdx.x < 64 && ((word >> threadIdx.x) & 1ull))
    s_site[__popcll(word & ((1ull << threadIdx.x) - 1ull))] = (unsigned char)threadIdx.x;
  __syncthreads();
  for (int e = threadIdx.x; e < n_active * C; e += 256) {
    const int k = e / C, c = e - k * C;
    const int site = s_site[k];
    const int oy = tile_y * 8 + (site >> 3), ox = tile_x * 8 + (site & 7);
    const size_t q = ((size_t)oy * p.g.w + ox) * C + c;
    if (p.dense) {
      float v = 0.0f;
      if (!p.zero_state) v = p.last_dense ? src[q] : z[q] + (((saved >> site) & 1ull) ? src[q] : 0.0f);
      out[q] = v;
      z[q] = v;
    } else {
      const float zo = z[q];
      const float inc = p.last_dense ? src[q] - zo : src[q];
      out[q] = inc;
      z[q] = zo + inc;
    }
  }
}

void launch_delay(const DelayParams& p, hipStream_t s) {
  hipLaunchKernelGGL(delay_kernel, dim3(p.g.tiles(), 1, p.st.n), dim3(256), 0, s, p);
}

__global__ __launch_bounds__(256) void copy_u64_kernel(uint64_t* dst, const uint64_t* src, size_t n, size_t stride) {
  const size_t so = (size_t)blockIdx.y * stride;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) at_stream(dst, so)[i] = at_stream(src, so)[i];
}

void launch_copy_u64(uint64_t* dst, const uint64_t* src, size_t n, Streams st, hipStream_t s) {
  hipLaunchKernelGGL(copy_u64_kernel, dim3((unsigned)((n + 255) / 256), st.n), dim3(256), 0, s, dst, src, n, st.stride);
}

// =============================================================================== ordered lists
// Workgroup (strip, set): strip = one row of tiles = 8 image rows.  Its first list position is
// the number of active sites in all earlier strips (a reduction over their occupancy words);
// inside the strip wave r owns image row r and scans the per-tile byte popcounts with a
// wave-wide prefix sum, so indices come out strictly ascending in y*W + x.
__global__ __launch_bounds__(512) void build_lists_kernel(const SetDesc* sets, size_t stream_stride) {
  __shared__ int s_part[8];
  __shared__ int s_rowcnt[8];
  SetDesc d = sets[blockIdx.y];  // the descriptors hold stream 0's pointers
  {
    const size_t so = (size_t)blockIdx.z * stream_stride;
    d.occ = at_stream(d.occ, so); d.idx = at_stream(d.idx, so);
    d.count = at_stream(d.count, so); d.bitmap = at_stream(d.bitmap, so);
  }
  const int strip = blockIdx.x;
  if (strip >= d.ty) return;
  const int tid = threadIdx.x, lane = tid & 63, r = tid >> 6;

  int cnt = 0;
  for (int t = tid; t < strip * d.tx; t += 512) cnt += __popcll(d.occ[t]);
  for (int o = 32; o > 0; o >>= 1) cnt += __shfl_down(cnt, o);
  if (lane == 0) s_part[r] = cnt;

  // row r of this strip: per-tile 8-bit masks
  int row_total = 0;
  for (int j0 = 0; j0 < d.tx; j0 += 64) {
    const int j = j0 + lane;
    const unsigned byte = j < d.tx ? (unsigned)((d.occ[strip * d.tx + j] >> (8 * r)) & 0xffull) : 0u;
    int c = __popc(byte);
    for (int o = 32; o > 0; o >>= 1) c += __shfl_down(c, o);
    row_total += __shfl(c, 0);
  }
  if (lane == 0) s_rowcnt[r] = row_total;
  __syncthreads();

  int base = 0;
  for (int i = 0; i < 8; ++i) base += s_part[i];
  int strip_total = 0;
  for (int i = 0; i < 8; ++i) {
    if (i < r) base += s_rowcnt[i];
    strip_total += s_rowcnt[i];
  }
  const int total_before = base;  // list position of the first active site of row r
  int running = total_before;
  const int y = strip * 8 + r;
  for (int j0 = 0; j0 < d.tx; j0 += 64) {
    const int j = j0 + lane;
    unsigned byte = j < d.tx ? (unsigned)((d.occ[strip * d.tx + j] >> (8 * r)) & 0xffull) : 0u;
    const int c = __popc(byte);
    int incl = c;  // inclusive wave scan
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o);
      if (lane >= o) incl += v;
    }
    int pos = running + incl - c;
    while (byte) {
      const int bit = __ffs(byte) - 1;
      byte &= byte - 1;
      d.idx[pos++] = y * d.w + j * 8 + bit;
    }
    running += __shfl(incl, 63);
  }
  if (strip == d.ty - 1 && tid == 0) {
    int s = 0;
    for (int i = 0; i < 8; ++i) s += s_part[i];
    *d.count = s + strip_total;
  }
  if (strip == 0) {  // tile bitmap: one ballot per 64 tiles
    const int n_tiles = d.tx * d.ty;
    for (int w0 = r * 64; w0 < n_tiles; w0 += 512) {
      const int t = w0 + lane;
      const uint64_t b = __ballot(t < n_tiles && d.occ[t] != 0);
      if (lane == 0) d.bitmap[w0 >> 6] = b;
    }
  }
}

void launch_build_lists(const SetDesc* sets_dev, int n_sets, int max_ty, Streams st, hipStream_t s) {
  hipLaunchKernelGGL(build_lists_kernel, dim3(max_ty, n_sets, st.n), dim3(512), 0, s, sets_dev, st.stride);
}

// =============================================================================== rounding step
// stage 1: block b sums the squares of its contiguous slice in a fixed order (thread-strided
// partials, then a shared-memory tree); stage 2: one block adds the kRmsBlocks partials the same
// way and writes k = tp * sqrt(sum / n) kept to 8 fraction bits.
__global__ __launch_bounds__(256) void rms_stage1_kernel(const float* x, size_t n, float* partial, size_t stream_stride) {
  x = at_stream(x, (size_t)blockIdx.y * stream_stride);
  partial = at_stream(partial, (size_t)blockIdx.y * stream_stride);
  __shared__ float s_sum[256];
  const size_t per = (n + kRmsBlocks - 1) / kRmsBlocks;
  const size_t lo = blockIdx.x * per, hi = min(n, lo + per);
  float acc = 0.0f;
  for (size_t i = lo + threadIdx.x; i < hi; i += 256) acc += x[i] * x[i];
  s_sum[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) s_sum[threadIdx.x] += s_sum[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = s_sum[0];
}
__global__ __launch_bounds__(256) void rms_stage2_kernel(const float* partial, size_t n, float tp, float* step_out,
                                                        size_t stream_stride) {
  partial = at_stream(partial, (size_t)blockIdx.y * stream_stride);
  step_out = at_stream(step_out, (size_t)blockIdx.y * stream_stride);
  __shared__ float s_sum[256];
  s_sum[threadIdx.x] = threadIdx.x < kRmsBlocks ? partial[threadIdx.x] : 0.0f;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) s_sum[threadIdx.x] += s_sum[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const float k = tp * sqrtf(s_sum[0] / (float)n);
    unsigned u = __float_as_uint(k);
    u = (u + 0x4000u) & 0xffff8000u;
    *step_out = __uint_as_float(u);
  }
}
void launch_rms_step(const float* x, size_t n, float tp, float* partial, float* step_out, Streams st, hipStream_t s) {
  static_assert(kRmsBlocks == 256, "stage 2 adds one partial per thread");
  hipLaunchKernelGGL(rms_stage1_kernel, dim3(kRmsBlocks, st.n), dim3(256), 0, s, x, n, partial, st.stride);
  hipLaunchKernelGGL(rms_stage2_kernel, dim3(1, st.n), dim3(256), 0, s, partial, n, tp, step_out, st.stride);
}

__global__ void fill_u64_kernel(uint64_t* p, size_t n, uint64_t v, size_t stream_stride) {
  p = at_stream(p, (size_t)blockIdx.y * stream_stride);
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
void launch_fill_u64(uint64_t* p, size_t n, uint64_t v, Streams st, hipStream_t s) {
  if (!n) return;
  int blocks = (int)((n + 255) / 256);
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(fill_u64_kernel, dim3(blocks, st.n), dim3(256), 0, s, p, n, v, st.stride);
}

}  // namespace evk
