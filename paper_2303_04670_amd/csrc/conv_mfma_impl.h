// Sparse incremental convolution on the matrix cores.
//
// Used where the per-tile channel contraction is a dense GEMM: c_in >= 9 (any count: the last
// channel chunk is zero-padded), c_out >= 16 (any count: the last block of 32 is zero-padded).
// Implicit GEMM per touched output tile (8 x 8 sites): M = 32 * MB sites (MB = 2: the whole
// tile as two 32-row MFMA blocks, rows 0-3 and 4-7; MB = 1: one workgroup per half tile),
// N = 32 output channels per workgroup (16 in the fp32 variant for launches that fill the chip
// unevenly, see NB below), K = taps x c_in.
//
//   fp32 mode : fp32 operands, v_mfma_f32_32x32x2_f32; a unit = one tap x 8 channels (4 MFMA
//               steps per block); MFMA j of a unit contracts channels {j, 4+j}: lanes 0-31 hold
//               channel j, lanes 32-63 channel 4+j, for both operands.
//   bf16 mode : the gather rounds increments to bf16 on their way into LDS, weights are bf16,
//               v_mfma_f32_32x32x16_bf16 with fp32 accumulation; a unit = one tap x 16 channels
//               (one MFMA per block); lanes 0-31 hold channels 0-7, lanes 32-63 channels 8-15.
//   split mode: fp32 accuracy from the bf16 matrix cores.  Each fp32 operand is written as
//               hi + lo with hi = bf16(x), lo = bf16(x - hi) (16 significant bits together); the
//               gather does that for the increments, the host for the weights; a product is
//               lo*hi + hi*lo + hi*hi, three bf16 MFMAs with fp32 accumulation (relative error of
//               a product about 2^-16, against 2^-8 in bf16 mode).  16 times the fp32 MFMA rate
//               at 3 MFMAs per product.
//
// Workgroup = NW (4 or 8) wavefronts that split K: the units of every channel chunk are dealt
// round-robin to the waves; each wave keeps the MB accumulators and the partial sums are added
// through LDS at the end.  K-splitting (rather than N-splitting), 8 waves and half tiles are what
// spread the low-resolution layers (24-88 tiles) over 256 CUs; the launcher picks MB and NW from
// the number of workgroups a layer yields.
//   Masks: the occupancy words of the input tiles under the halo are turned into one bit row per
//     patch row in LDS; the touched word of the tile and the gather predicates come from those.
//   A operand: the input halo patch of the current chunk, gathered once per workgroup into LDS
//     with buffer loads whose offset is pushed out of range for inactive / out-of-image sites:
//     the hardware bounds check returns zeros without a memory access (conditioned fetch).  The
//     next chunk's patch is fetched into registers while the current one is being contracted.
//     A lane reads its fragment with one ds_read_b128; the LDS site stride keeps that
//     conflict-free for stride-1 layers.
//   B operand: weights re-laid as [tap][c_in/4][c_out][4] (fp32) or [tap][c_in/8][c_out][8]
//     (bf16) so that a lane's fragment is one 16-byte buffer load (L2-resident), held in a
//     three-register ring two units ahead, across chunk boundaries.
// Epilogue: lane = output channel, so every z / increment access is a 128-byte row segment; the
// old z values are requested before the contraction starts.  ADD nodes that consume the conv
// output (residual add + activation, skip adds) run here as well, writing their own buffers.
//
// A bilinear x2 up-sampling in front of the conv (Eq.9-10: both linear) never exists in memory
// (UPS variants).  Along the image border the patch is interpolated from the stored tensor on
// its way into LDS.  Away from the border the up-sampling is folded into the weights: the
// outputs of one phase (row parity, column parity) are a conv of the stored tensor with fewer
// taps (4 x 4 for 5 x 5), so a workgroup takes one phase of one tile of stored sites, gathers
// the stored tensor directly and writes its 64 outputs two sites apart.  Which workgroup does
// which is read from a list made at set-up (ConvParams::fold_list).
//
// The fp32 matrix instruction executes on the SIMD's vector pipeline: a vector instruction of any
// wave of the SIMD takes time from the MFMAs.  Hence the addressing style throughout: per-lane
// parts of an address are computed once and kept, per-unit / per-row parts live in scalar
// registers (buffer instructions with a scalar offset), masks are tested where their bits sit.
// (This header holds the kernel template and its launchers; one translation unit per operand
// mode instantiates it, so that the three modes compile in parallel.)
#pragma once
#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "evconv_kernels.h"

namespace evk {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
// Phase stamps.  In a build with -DEVCONV_PHASE_STAMPS (never the product build) one lane per
// workgroup writes the 100 MHz wall clock at the boundaries of the kernel's phases into a device
// array of the translation unit; evconv_debug_phase_stamps copies the records out.  Without the
// define EVK_PHASE expands to nothing.  A record is 32 x u64:
enum PhaseField {
  kPhStart = 0,            // first instruction of the workgroup
  kPhOccInLds = 1,         // occupancy words arrived and in LDS (the gather addressing is worked out meanwhile)
  kPhBitRows = 2,          // bit rows of the patch built
  kPhAddressed = 3,        // touched words, old z requested, gather offsets conditioned
  kPhFirstIssued = 4,      // first patch chunk and first weight fragments requested
  kPhFirstPatchInLds = 5,  // first chunk arrived, in LDS (and interpolated), next chunk requested
  kPhChunksDone = 6,       // end of the chunk loop
  kPhFusedRequested = 10,  // operands of the fused stages requested
  kPhReduced = 7,          // partial sums of the waves in LDS
  kPhArrived = 14,         // everything requested so far has arrived
  kPhEpilogueDone = 8,     // all passes of the epilogue issued
  kPhFlagsBallot = 11,     // (start of the nonzero-flag collection)
  kPhFlagsInLds = 12,      // the waves' flag words written
  kPhFlagsBarrier = 13,    // ... and visible to the workgroup
  kPhEnd = 9,              // tile words OR-ed into memory
  kPhContractionTicks = 20,  // ticks inside the contraction loops, all chunks
  kPhChunkChangeTicks = 21,  // ticks in barriers, LDS stores and interpolation between them
  kPhGrid = 24, kPhBlock = 25, kPhHwId = 26,  // workgroups of the launch, this one's index, HW_ID | XCC_ID << 32
  kPhLayer = 27,           // output height | c_in << 16 | k << 32 | c_out << 40
};
#ifdef EVCONV_PHASE_STAMPS
constexpr unsigned kPhaseRecords = 1u << 15;
static __device__ unsigned long long g_phase[kPhaseRecords][32];
static __device__ unsigned g_phase_n;
#define EVK_PHASE(i) do { if (tid == 0 && ph_slot < kPhaseRecords) g_phase[ph_slot][i] = wall_clock64(); } while (0)
#else
#define EVK_PHASE(i) do {} while (0)
#endif
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// operand modes of the contraction
constexpr int kOpF32 = 0;    // fp32 operands, v_mfma_f32_32x32x2_f32
constexpr int kOpBf16 = 1;   // bf16 operands (increments rounded in the gather), v_mfma_f32_32x32x16_bf16
constexpr int kOpSplit = 2;  // fp32 operands split into bf16 high + low parts, three bf16 MFMAs per product

// one weight fragment of a lane; .l is the low-part plane in split mode, unused otherwise
struct BFrag { float4 h, l; };
// one patch fragment of a lane: both 32-row blocks (h1: second block, two-block workgroups only)
// and their low parts (split mode only)
struct AFrag { float4 h0, h1, l0, l1; };

__device__ __forceinline__ float act_m(int act, float v) {
  if (act == kActRelu) return fmaxf(v, 0.0f);
  if (act == kActSigmoid) return 1.0f / (1.0f + expf(-v));
  if (act == kActTanh) return tanhf(v);
  if (act == kActOneMinus) return 1.0f - v;
  return v;
}

// fp32 -> bf16, round to nearest even, two values packed low/high: one v_cvt_pk_bf16_f32
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  floatx2 v;
  v.x = lo;
  v.y = hi;
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// Largest halo patch (sites) a variant can meet: 64- and 128-channel chunks are used with stride 1
// and taps <= 3, 32-channel chunks with stride 1 (taps <= 7), 16-channel chunks also with stride 2.
constexpr int max_patch_sites(int chunk, int mb) {
  const int rows = 4 * mb - 1;
  return chunk >= 64 ? (rows + 3) * 10 : chunk == 32 ? (rows + 7) * 14 : (rows * 2 + 7) * 21;
}

// The register budget is held to 4 (half tiles) or 3 (whole tiles) waves per SIMD: the bf16 and
// split modes are bound by latencies, not by the matrix cores, and lose a third of their speed
// when one workgroup fewer fits on a CU.
//
// UPS: the conv's input is the bilinear x2 up-sampling of p.in (half-pixel centres, weights
// 0.25 / 0.75, clamped borders), which is never written to memory: the low-resolution sites under
// the halo are gathered into a second LDS buffer and every patch element is interpolated from
// four of them on its way into the patch buffer.  p.gi describes the up-sampled tensor, p.lo_h x
// p.lo_w the stored one; p.occ_in are the stored tensor's occupancy words, and an up-sampled
// site is active where one of its four sources is.
// NB: output channels per workgroup.  32 is the normal shape.  16 (fp32, half tiles, no up-sampling)
// is for launches that would otherwise leave the chip unevenly filled: the same half tile as two
// 16-row blocks of v_mfma_f32_16x16x4_f32 (a unit = one tap x 16 channels, MFMA j of a unit
// contracts channels {j, 4+j, 8+j, 12+j}: lanes 16 q .. 16 q + 15 hold channel 4 q + j), twice the
// workgroups at half the work each.
template <int CHUNK, int NW, int OPM, int MB, bool UPS, int NB = 32>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NB == 16 ? 4 : MB == 1 && !(UPS && NW == 4) ? 4 : 3)))
void conv_mfma_kernel(ConvParams p) {
  // this workgroup's stream: every state pointer of p is used through at_stream(.., so); p itself
  // stays untouched so that it remains in the kernel-argument segment
  const size_t so = (size_t)blockIdx.z * p.st.stride;
  constexpr bool BF16 = OPM != kOpF32;     // bf16 MFMA, 16 channels per unit
  constexpr bool SPLIT = OPM == kOpSplit;  // operands as bf16 high + low parts, three products
  constexpr int NT = NW * 64;
  // LDS site stride in 4-byte words; stride / 4 is odd (the eight sites of a patch row fall into
  // eight distinct 16-byte slots of the banks).  Split mode keeps a high plane and a low plane of
  // CHUNK bf16 each per site.
  constexpr int CS = (BF16 && !SPLIT) ? CHUNK / 2 + 4 : CHUNK + 4;
  constexpr int LO = CHUNK / 2;  // word offset of the low plane inside a site (split mode)
  static_assert(NB == 32 || (NB == 16 && OPM == kOpF32 && MB == 1 && !UPS), "16-channel blocks: fp32 half tiles only");
  constexpr int UCH = (BF16 || NB == 16) ? 16 : 8;  // channels per unit
  constexpr int KG = CHUNK / UCH;     // units per tap and chunk
  constexpr int NV = CHUNK / 4;       // float4 per patch site
  constexpr int MAXV = (max_patch_sites(CHUNK, MB) * NV + NT - 1) / NT;  // patch float4 per thread
  constexpr int SUBS = 2 / MB;        // workgroups per tile
  constexpr int NROWS = 4 * MB;       // output rows of this workgroup
  constexpr int NSITES = 32 * MB;
  constexpr int EP_SITES = NT / NB;   // sites per epilogue pass
  constexpr int EP_ITERS = NSITES / EP_SITES;
  static_assert(EP_ITERS >= 1 && EP_SITES <= 32, "epilogue mapping");
  constexpr int NACC = NB == 16 ? 8 : MB * 16;  // accumulator registers of a lane
  constexpr int SLOT = NACC * 64;     // floats per partial-sum slot
  constexpr int CSL = CHUNK + 4;      // UPS: site stride of the low-resolution fp32 buffer
  constexpr int LPMAX = 10;           // UPS: a 14-row patch has sources in at most 14 / 2 + 3 rows
  constexpr int MAXG = UPS ? (LPMAX * LPMAX * NV + NT - 1) / NT : MAXV;  // gathered float4 per thread
  // a weight-folded workgroup gathers an (NROWS + 3) x 11 patch (4 x 4 taps) through the same registers
  static_assert(!UPS || MAXG * NT >= (4 * MB + 3) * 11 * NV, "folded patch does not fit the gather registers");
  extern __shared__ __align__(16) float s_mem[];
  __shared__ uint64_t s_occ[16];
  __shared__ unsigned s_rows[24];  // bit px of s_rows[py]: patch site (py, px) is active
  __shared__ unsigned s_lrows[UPS ? LPMAX : 1];  // UPS: the same for the low-resolution source region
  __shared__ uint64_t s_nz[(2 + kMaxFusedAdds) * NW];  // nonzero-site bits per wave: conv, each fused ADD, fused sparsification
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#ifdef EVCONV_PHASE_STAMPS
  unsigned ph_slot = 0xffffffffu;
  if (tid == 0) {
    ph_slot = atomicAdd(&g_phase_n, 1u);
    if (ph_slot < kPhaseRecords) {
      unsigned long long* r = g_phase[ph_slot];
      for (int i = 1; i < 24; ++i) r[i] = 0;
      r[kPhGrid] = (unsigned long long)gridDim.x * gridDim.y;
      r[kPhBlock] = blockIdx.x + (unsigned long long)blockIdx.y * gridDim.x;
      r[kPhHwId] = __builtin_amdgcn_s_getreg(4 | (31 << 11)) | ((unsigned long long)__builtin_amdgcn_s_getreg(20 | (31 << 11)) << 32);
      r[kPhLayer] = (unsigned long long)p.go.h | ((unsigned long long)p.gi.c << 16) | ((unsigned long long)p.k << 32) |
                    ((unsigned long long)p.go.c << 40);
    }
  }
#endif
  EVK_PHASE(kPhStart);
  // Consecutive workgroups (x fastest) go to the chip's 8 XCDs in turn, each with an L2 of its own.
  // x over tiles: an XCD sees every eighth tile and all of the weights; x over the blocks of
  // output channels (wg_swap): an XCD sees all tiles and one in eight (four, two) of the weight
  // blocks.  The launcher picks whichever of the two operands is larger to be split.
  const int wg_tile = p.wg_swap ? blockIdx.y : blockIdx.x, wg_co = p.wg_swap ? blockIdx.x : blockIdx.y;
  int tile = wg_tile / SUBS;
  const int sub = wg_tile % SUBS;
  // Weight-folded workgroup (UPS variants with a fold list): its 8 x 8 "tile" is a tile of stored
  // sites, its outputs are the up-sampled sites of one phase, (2 * row + fpy, 2 * column + fpx);
  // it gathers the stored tensor directly (no interpolation) under a fold_k x fold_k window that
  // starts fold_base[parity] rows / columns from the site, and takes that phase's weight set.
  bool fold = false;
  int fpy = 0, fpx = 0;
  if (UPS && OPM != kOpBf16 && p.fold_list) {  // (never used with bf16-declared weights)
    const int e = p.fold_list[tile];
    tile = e;
    if (e < 0) {
      fold = true;
      tile = (-1 - e) >> 2;
      fpy = ((-1 - e) >> 1) & 1;
      fpx = (-1 - e) & 1;
    }
  }
  const bool ups = UPS && !fold;  // this workgroup interpolates its patch
  const int r0 = sub * NROWS;  // first tile row of this workgroup
  const uint64_t row_mask = MB == 2 ? ~0ull : (0xffffffffull << (32 * sub));
  const int n_tx = fold ? (p.lo_w + 7) >> 3 : p.go.tx;
  const int tile_y = tile / n_tx, tile_x = tile - tile_y * n_tx;
  const int s = p.stride, K = fold ? p.fold_k : p.k;
  const int H = p.gi.h, W = p.gi.w, Cin = p.gi.c, Cout = p.go.c;
  const int iy0 = fold ? tile_y * 8 + r0 + p.fold_base[fpy] : (tile_y * 8 + r0) * s - p.pad;
  const int ix0 = fold ? tile_x * 8 + p.fold_base[fpx] : tile_x * 8 * s - p.pad;
  const int PH = (NROWS - 1) * s + K, PW = 7 * s + K;
  // The region whose stored occupancy is read: the patch itself, or (UPS) the low-resolution
  // sources of the patch: rows (iy0 >> 1) - 1 .. and columns likewise, PH / 2 + 3 by PW / 2 + 3
  // sites (a source index is i/2 - 1, i/2 or i/2 + 1 before clamping to the image).
  const int SH = UPS ? p.lo_h : H, SW = UPS ? p.lo_w : W;  // stored tensor
  const int s_ty = (SH + 7) >> 3, s_tx = (SW + 7) >> 3;
  const int gy0 = ups ? (iy0 >> 1) - 1 : iy0, gx0 = ups ? (ix0 >> 1) - 1 : ix0;
  const int GH = ups ? PH / 2 + 3 : PH, GW = ups ? PW / 2 + 3 : PW;
  const int rty0 = gy0 >> 3, rtx0 = gx0 >> 3;
  const int rny = ((gy0 + GH - 1) >> 3) - rty0 + 1, rnx = ((gx0 + GW - 1) >> 3) - rtx0 + 1;

  // occupancy words of the fused ADD nodes' other inputs: requested first, so that their latency
  // runs alongside that of the input's occupancy words instead of after it
  uint64_t skip_raw[kMaxFusedAdds];
#pragma unroll
  for (int f = 0; f < kMaxFusedAdds; ++f) {
    skip_raw[f] = 0;
    if (f >= p.n_fused || p.dense) continue;
    if (fold) {
      // per lane (= site of the stored tile) the word of the up-sampled tile its output lies in;
      // turned into this phase's site bits further down
      const int ly = lane >> 3, lx = lane & 7;
      skip_raw[f] = at_stream(p.fused[f].occ_skip, so)[(2 * tile_y + (ly >> 2)) * p.go.tx + 2 * tile_x + (lx >> 2)];
    } else {
      skip_raw[f] = at_stream(p.fused[f].occ_skip, so)[tile];
    }
  }
  uint64_t occ_w = 0;
  if (tid < 16) {
    const int ry = tid >> 2, rx = tid & 3;
    const int ty = rty0 + ry, tx = rtx0 + rx;
    if (ry < rny && rx < rnx && ty >= 0 && ty < s_ty && tx >= 0 && tx < s_tx)
      occ_w = p.dense ? ~0ull : at_stream(p.occ_in, so)[ty * s_tx + tx];
  }

  // While the occupancy words are on their way: everything about the gather that depends on the
  // tile's position only.
  // ---- patch gather: per thread a fixed list of (LDS offset, byte offset into the input)
  // The gathered region is the patch itself, or (UPS) its low-resolution source region, which
  // goes to a second fp32 buffer behind the patch buffer.
  constexpr unsigned kOob = 0x80000000u;
  // Row pitch of the patch in LDS (4-byte words).  The LDS serves a 16-byte read per lane in
  // groups of 16 lanes over 64 banks; the 16 lanes of an A-fragment read are two rows of eight
  // sites.  The site stride (an odd number of 16-byte slots) spreads a row's eight sites over
  // eight distinct slots; a row pitch of 128 bytes modulo 256 puts the next row's sites on the
  // other eight.  (Stride-2 layers read every other site and row: no pitch frees them of
  // conflicts, they keep the dense pitch.)
  const int RP = s == 1 ? ((PW * CS + 31) / 64) * 64 + 32 : PW * CS;
  float* const s_low = s_mem + PH * RP;  // UPS only
  const int total_v = GH * GW * NV;
  const int gw_magic = (65536 + GW - 1) / GW;  // site / GW == (site * gw_magic) >> 16 for site < 441
  int lds_off[MAXG];     // (until the occupancy is known: patch row and column in bits 16-23 and 24-31)
  unsigned g_off[MAXG];
#pragma unroll
  for (int j = 0; j < MAXG; ++j) {
    const int e = tid + j * NT;
    lds_off[j] = -1;
    g_off[j] = kOob;
    if (e < total_v) {
      const int site = e / NV, v = e - site * NV;
      const int py = (site * gw_magic) >> 16, px = site - py * GW;
      lds_off[j] = (ups ? site * CSL + v * 4 : py * RP + px * CS + v * (BF16 ? 2 : 4)) | (py << 16) | (px << 24);
      g_off[j] = (unsigned)((((gy0 + py) * SW + gx0 + px) * Cin + v * 4) * 4);
    }
  }
  // UPS: every patch element from its four sources in the low-resolution buffer, with the
  // weights and the summation order of the stand-alone up-sampling operator
  //
  // Work item = one 2 x 2 block of up-sampled sites (rows 2i+1, 2i+2, columns 2j+1, 2j+2) x four
  // channels: its four values come from the same four stored sites (rows i, i+1, columns j, j+1,
  // clamped to the image), so the four reads and the two horizontal sums per stored row are
  // shared; a site without an active source comes out as zero because inactive sources are
  // stored as zeros.  The items of a thread are the same for every chunk: offsets and masks are
  // worked out once (this arithmetic would otherwise take vector-ALU time from the fp32 matrix
  // instructions, which run on the same pipeline).
  constexpr int MAXB = UPS ? (8 * (MB == 2 ? 8 : 6) * NV + NT - 1) / NT : 1;  // <= 8 x 8 blocks (K <= 7)
  // per item two packed words: ib_src = source offset (12 bits) | row step (10) | column step (6);
  // ib_dst = patch offset + 4096 (16 bits) | write mask (4) | inside-the-image mask (4)
  int ib_src[MAXB], ib_dst[MAXB];
#pragma unroll
  for (int b = 0; b < MAXB; ++b) ib_src[b] = ib_dst[b] = 0;
  if (ups) {
    const int by0 = (iy0 - 1) >> 1, bx0 = (ix0 - 1) >> 1;
    const int nby = ((iy0 + PH - 2) >> 1) - by0 + 1, nbx = ((ix0 + PW - 2) >> 1) - bx0 + 1;
    const int nbx_magic = (65536 + nbx - 1) / nbx;  // blk / nbx == (blk * nbx_magic) >> 16 for blk < 64
#pragma unroll
    for (int b = 0; b < MAXB; ++b) {
      const int e = tid + b * NT;
      const int blk = e / NV, v = e - blk * NV;
      ib_src[b] = ib_dst[b] = 0;
      if (blk < nby * nbx) {
        const int bi = (blk * nbx_magic) >> 16, bj = blk - bi * nbx;
        const int i = by0 + bi, j = bx0 + bj;
        const int cy0 = min(max(i, 0), SH - 1), cy1 = min(max(i + 1, 0), SH - 1);
        const int cx0 = min(max(j, 0), SW - 1), cx1 = min(max(j + 1, 0), SW - 1);
        ib_src[b] = (((cy0 - gy0) * GW + (cx0 - gx0)) * CSL + v * 4) | (((cy1 - cy0) * GW * CSL) << 12) |
                    (((cx1 - cx0) * CSL) << 22);
        const int py = 2 * i + 1 - iy0, px = 2 * j + 1 - ix0;  // patch coordinates of the block, -1 at least
        const int dst = py * RP + px * CS + v * (BF16 ? 2 : 4) + 4096;
        int mask = 0;
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
          for (int c = 0; c < 2; ++c) {
            const bool in_patch = py + r >= 0 && py + r < PH && px + c >= 0 && px + c < PW;
            const bool in_image = (unsigned)(iy0 + py + r) < (unsigned)H && (unsigned)(ix0 + px + c) < (unsigned)W;
            if (in_patch) mask |= 1 << (r * 2 + c);
            if (in_patch && in_image) mask |= 16 << (r * 2 + c);
          }
        ib_dst[b] = dst | (mask << 16);
      }
    }
  }

  if (tid < 16) s_occ[tid] = occ_w;
  __syncthreads();
  EVK_PHASE(kPhOccInLds);
  if (tid < GH) {  // one bit row per row of the region; out-of-image sites are 0
    const int gy = gy0 + tid;
    unsigned bits = 0;
    if ((unsigned)gy < (unsigned)SH) {
      const int ry = (gy >> 3) - rty0;
      // 32 consecutive columns starting at image column rtx0 * 8
      uint64_t span = 0;
#pragma unroll
      for (int rx = 0; rx < 4; ++rx)
        span |= ((s_occ[ry * 4 + rx] >> ((gy & 7) * 8)) & 0xffull) << (8 * rx);
      bits = (unsigned)(span >> (gx0 - rtx0 * 8));
      // clear columns outside the image (dense mode sets every bit) and beyond the region
      const int lo = max(0, -gx0), hi = min(GW, SW - gx0);  // valid columns in [lo, hi)
      unsigned m = hi >= 32 ? ~0u : ((1u << max(hi, 0)) - 1u);
      m &= ~((1u << lo) - 1u);
      bits &= m;
    }
    if (ups) s_lrows[tid] = bits; else s_rows[tid] = bits;
  }
  __syncthreads();
  if (ups) {
    // an up-sampled site is active where one of its four sources is: OR of two source rows, then
    // of two source columns; sites outside the up-sampled image stay 0
    if (tid < PH) {
      const int iy = iy0 + tid;
      unsigned bits = 0;
      if ((unsigned)iy < (unsigned)H) {
        const int hy = iy >> 1;
        const int y0 = (iy & 1) ? hy : max(hy - 1, 0), y1 = (iy & 1) ? min(hy + 1, SH - 1) : hy;
        const unsigned src = s_lrows[y0 - gy0] | s_lrows[y1 - gy0];
        for (int px = 0; px < PW; ++px) {
          const int ix = ix0 + px;
          if ((unsigned)ix >= (unsigned)W) continue;
          const int hx = ix >> 1;
          const int x0 = (ix & 1) ? hx : max(hx - 1, 0), x1 = (ix & 1) ? min(hx + 1, SW - 1) : hx;
          bits |= (((src >> (x0 - gx0)) | (src >> (x1 - gx0))) & 1u) << px;
        }
      }
      s_rows[tid] = bits;
    }
    __syncthreads();
  }

  EVK_PHASE(kPhBitRows);
  // touched word of this workgroup's rows (identical in all waves): OR of the K bit rows under a
  // site, then any of the K columns
  uint64_t touched_word;
  {
    const int ly = lane >> 3, lx = lane & 7;
    const int oy = tile_y * 8 + ly, ox = tile_x * 8 + lx;
    const int lr = ly - r0;
    bool touched = false;
    // (a weight-folded workgroup's tile lies inside the stored image, all of its outputs exist)
    if (lr >= 0 && lr < NROWS && (fold || (oy < p.go.h && ox < p.go.w))) {
      unsigned rows = 0;
      for (int ky = 0; ky < K; ++ky) rows |= s_rows[lr * s + ky];
      touched = p.dense || ((rows >> (lx * s)) & ((1u << K) - 1u)) != 0;
    }
    touched_word = __ballot(touched);
  }
  // fused ADD nodes: their other input may be active where the conv is not
  uint64_t skip_word[kMaxFusedAdds];
  uint64_t site_word = touched_word;  // sites this workgroup has to visit in the epilogue
#pragma unroll
  for (int f = 0; f < kMaxFusedAdds; ++f) {
    skip_word[f] = 0;
    if (f < p.n_fused && fold && !p.dense)
      skip_raw[f] = __ballot(((skip_raw[f] >> ((2 * ((lane >> 3) & 3) + fpy) * 8 + 2 * (lane & 3) + fpx)) & 1ull) != 0);
    if (f < p.n_fused) skip_word[f] = p.dense ? touched_word : (skip_raw[f] & row_mask);
    site_word |= skip_word[f];
  }
  if (site_word == 0) return;
  const bool conv_on = touched_word != 0;

  // Epilogue addressing.  Thread = output channel co0 + tid % 32 at the EP_ITERS sites
  // r0 * 8 + it * EP_SITES + tid / 32 (EP_SITES = 8 or 16: consecutive `it` are one or two tile rows
  // apart).  Every tensor of the output geometry is reached as buffer + the byte offset of the
  // thread's first site (one vector register for the whole kernel) + a scalar offset per `it`;
  // an access that must not happen gets an out-of-range vector offset (loads return 0, stores are
  // dropped).  The bits of a thread's sites are kept where they are in the 64-bit words, EP_SITES
  // bits apart: no per-site shifts, no 64-bit address arithmetic on the vector ALU.
  const int co = tid & (NB - 1);
  const int co0 = wg_co * NB;
  const int es = tid / NB;
  // (weight-folded: site (y, x) of the stored tile is output site (2y + fpy, 2x + fpx))
  const int ey = tile_y * 8 + r0 + (es >> 3), ex = tile_x * 8 + (es & 7);
  const unsigned ep_voff =
      (unsigned)((((fold ? 2 * ey + fpy : ey) * p.go.w + (fold ? 2 * ex + fpx : ex)) * Cout + co0 + co) * 4);
  const unsigned ep_step = (unsigned)((EP_SITES / 8) * p.go.w * Cout * 4) << (fold ? 1 : 0);
  const int out_bytes = p.go.h * p.go.w * Cout * 4;
  constexpr unsigned kSkipAccess = 0x80000000u;
  constexpr uint64_t kMine = EP_SITES == 8 ? 0x0101010101010101ull : EP_SITES == 16 ? 0x0001000100010001ull : 0x1ull;
  // c_out need not be a multiple of 32: the last block's weights are zero-padded and the threads
  // of the channels that do not exist own no sites (they take no part in the epilogue)
  const bool co_ok = co0 + co < Cout;
  auto mine = [&](uint64_t w) { return co_ok ? (w >> (r0 * 8 + es)) & kMine : 0ull; };   // bit it * EP_SITES: site `it`
  auto has = [&](uint64_t sp, int it) { return ((sp >> (it * EP_SITES)) & 1ull) != 0; };
  auto out_rsrc = [&](const void* ptr) {
    return __builtin_amdgcn_make_buffer_rsrc((void*)ptr, 0, out_bytes, 0x00020000);
  };
  auto ep_load = [&](const __amdgpu_buffer_rsrc_t& r, bool on, int it) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, on ? ep_voff : kSkipAccess, it * ep_step, 0));
  };
  const uint64_t touched_mine = mine(touched_word), site_mine = mine(site_word);
  const __amdgpu_buffer_rsrc_t z_rsrc = out_rsrc(at_stream(p.z, so));

  // old z values of the epilogue, requested now so that they arrive during the contraction
  float z_old[EP_ITERS];
#pragma unroll
  for (int it = 0; it < EP_ITERS; ++it) z_old[it] = ep_load(z_rsrc, !p.dense && has(touched_mine, it), it);

  // the gather's offsets, now conditioned on the occupancy (out of range where the site is inactive)
#pragma unroll
  for (int j = 0; j < MAXG; ++j) {
    if (lds_off[j] < 0) continue;
    const int py = (lds_off[j] >> 16) & 0xff, px = lds_off[j] >> 24;
    lds_off[j] &= 0xffff;
    const unsigned row = ups ? s_lrows[py] : s_rows[py];
    if (!((row >> px) & 1u)) g_off[j] = kOob;
  }
  // c_in need not be a multiple of four: the 16-byte load of a site's last channel group then
  // runs into the next site (buffer loads of dwords need dword alignment only); the foreign
  // components are zeroed on the way into LDS.  The range is extended by those 12 bytes so that
  // the last site's group is not rejected as a whole (every tensor of the workspace is followed
  // by padding or by another buffer of the workspace).
  const int tail = Cin & 3;
  const __amdgpu_buffer_rsrc_t in_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)at_stream(p.in, so), 0, SH * SW * Cin * 4 + (tail ? 12 : 0), 0x00020000);
  float4 pre[MAXG];
  // c_in need not be a multiple of the chunk: channel groups beyond c_in read as zeros (their
  // weight rows are zero padding as well)
  const bool ragged = (Cin % CHUNK) != 0;
  auto fetch = [&](int c0) {
#pragma unroll
    for (int j = 0; j < MAXG; ++j) {
      unsigned off = g_off[j];
      if (ragged && c0 + ((tid + j * NT) % NV) * 4 >= Cin) off = kOob;
      pre[j] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(in_rsrc, off, c0 * 4, 0));
    }
  };
  // one float4 of patch channels into the patch buffer, in the operand mode's format
  auto put = [&](int off, const float4& x) {
    if (SPLIT) {
      // x = hi + lo + O(2^-17 |x|): hi = bf16(x), lo = bf16(x - hi)
      uint2 h, l;
      h.x = pack_bf16x2(x.x, x.y);
      h.y = pack_bf16x2(x.z, x.w);
      l.x = pack_bf16x2(x.x - __uint_as_float(h.x << 16), x.y - __uint_as_float(h.x & 0xffff0000u));
      l.y = pack_bf16x2(x.z - __uint_as_float(h.y << 16), x.w - __uint_as_float(h.y & 0xffff0000u));
      *(uint2*)&s_mem[off] = h;
      *(uint2*)&s_mem[off + LO] = l;
    } else if (BF16) {
      uint2 w;
      w.x = pack_bf16x2(x.x, x.y);
      w.y = pack_bf16x2(x.z, x.w);
      *(uint2*)&s_mem[off] = w;
    } else {
      *(float4*)&s_mem[off] = x;
    }
  };
  auto stash = [&](int c0) {
    if (tail) {  // (uniform; nets with c_in % 4 == 0 pay nothing)
#pragma unroll
      for (int j = 0; j < MAXG; ++j) {
        const int left = Cin - (c0 + ((tid + j * NT) % NV) * 4);  // channels of this group inside c_in
        if (left > 0 && left < 4) {
          if (left < 2) pre[j].y = 0.0f;
          if (left < 3) pre[j].z = 0.0f;
          pre[j].w = 0.0f;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < MAXG; ++j)
      if (lds_off[j] >= 0) {
        if (ups) *(float4*)&s_low[lds_off[j]] = pre[j];
        else put(lds_off[j], pre[j]);
      }
  };
  auto interpolate = [&]() {
#pragma unroll
    for (int b = 0; b < MAXB; ++b) {
      const int mask = ib_dst[b] >> 16;
      if (mask == 0) continue;
      const float* q = &s_low[ib_src[b] & 0xfff];
      const int dy = (ib_src[b] >> 12) & 0x3ff, dx = ib_src[b] >> 22;
      const float4 v00 = *(const float4*)q, v01 = *(const float4*)(q + dx);
      const float4 v10 = *(const float4*)(q + dy), v11 = *(const float4*)(q + dy + dx);
      // horizontal sums of the two stored rows for the odd (a) and the even (b) column, then the
      // vertical ones: the same products and order as wy0 * (wx0 * v00 + wx1 * v01) + wy1 * (...)
      auto hsum = [](float w0, const float4& l, float w1, const float4& r) {
        return make_float4(w0 * l.x + w1 * r.x, w0 * l.y + w1 * r.y, w0 * l.z + w1 * r.z, w0 * l.w + w1 * r.w);
      };
      const float4 a0 = hsum(0.75f, v00, 0.25f, v01), b0 = hsum(0.25f, v00, 0.75f, v01);
      const float4 a1 = hsum(0.75f, v10, 0.25f, v11), b1 = hsum(0.25f, v10, 0.75f, v11);
      const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
      const int dst = (ib_dst[b] & 0xffff) - 4096;
      if (mask & 1) put(dst, (mask & 16) ? hsum(0.75f, a0, 0.25f, a1) : zero);
      if (mask & 2) put(dst + CS, (mask & 32) ? hsum(0.75f, b0, 0.25f, b1) : zero);
      if (mask & 4) put(dst + RP, (mask & 64) ? hsum(0.25f, a0, 0.75f, a1) : zero);
      if (mask & 8) put(dst + RP + CS, (mask & 128) ? hsum(0.25f, b0, 0.75f, b1) : zero);
    }
  };

  floatx16 acc0, acc1;
#pragma unroll
  for (int i = 0; i < 16; ++i) { acc0[i] = 0.0f; acc1[i] = 0.0f; }
  floatx4 c16a = {0.f, 0.f, 0.f, 0.f}, c16b = {0.f, 0.f, 0.f, 0.f};  // NB == 16: the two 16-row blocks
  // operand lane: k-group `half` (two groups of 32 lanes, or four of 16), row / column m of the block
  const int half = NB == 16 ? lane >> 4 : lane >> 5, m = NB == 16 ? lane & 15 : lane & 31;
  const int mly = m >> 3, mlx = m & 7;  // site of this lane inside a block
  const int cop = p.c_out_pad;
  const int n_units = K * K * KG;
  const int cin_pad = (Cin + CHUNK - 1) / CHUNK * CHUNK;    // the weights are zero-padded to whole chunks
  const int cin_rows = BF16 ? cin_pad >> 3 : cin_pad >> 2;  // 16-byte weight rows per tap: 8 bf16 or 4 floats
  const int a_lane_off = mly * s * RP + mlx * s * CS + half * 4;
  const int a_blk1 = (NB == 16 ? 2 : 4) * s * RP;  // the second block starts four (two) tile rows further down
  // units of this wave: u_j = wave + j * NW, j < n_mine
  const int n_mine = (n_units - wave + NW - 1) / NW;
  const int last = n_mine - 1;
  const int k_magic = (65536 + K - 1) / K;  // tap / K == (tap * k_magic) >> 16 for tap < 49

  // Both fragment addresses are a per-lane constant plus a per-unit part that is the same in all
  // lanes; the latter is kept in scalar registers (pinned there with readfirstlane), so that a
  // unit costs one vector add: vector-ALU time is taken from the fp32 matrix instructions.
  // B: buffer load with the lane part as vector offset and the unit part as scalar offset
  // (bytes; the launcher checks that the re-laid weights stay below 2 GiB).
  const unsigned w_plane = (unsigned)(K * K * cin_rows * cop) * 16u;  // split mode: the low-part plane follows
  const unsigned w_set = w_plane * (SPLIT ? 2u : 1u);  // one weight set; a folded workgroup takes its phase's
  const char* const w_base = fold ? (const char*)p.w_fold + (size_t)(fpy * 2 + fpx) * w_set : (const char*)p.w;
  const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)w_base, 0, (int)w_set, 0x00020000);
  const unsigned w_lane = (unsigned)(half * cop + co0 + m) * 16u;
  // unit j of the chunk starting at channel c0 (j clamped to the last unit so that look-ahead
  // loads stay unconditional and in bounds)
  auto b_load = [&](int c0, int j) {
    const int u = wave + min(j, last) * NW;
    const int tap = u / KG, kg = u % KG;
    const int row0 = BF16 ? (c0 >> 3) : (c0 >> 2);
    constexpr int kRowsPerUnit = BF16 ? UCH / 8 : UCH / 4;  // 16-byte weight rows of a unit
    const unsigned soff = (unsigned)__builtin_amdgcn_readfirstlane(((tap * cin_rows + row0 + kg * kRowsPerUnit) * cop) << 4);
    BFrag f;
    f.h = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, w_lane, soff, 0));
    f.l = SPLIT ? __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, w_lane, soff + w_plane, 0)) : f.h;
    return f;
  };
  // ... and LDS offset of its A fragment
  auto a_off = [&](int j) {
    const int u = wave + j * NW;
    const int tap = u / KG, kg = u % KG;
    const int ky = (tap * k_magic) >> 16, kx = tap - ky * K;
    return a_lane_off + __builtin_amdgcn_readfirstlane(ky * RP + kx * CS + kg * (NB == 16 ? 16 : 8));  // words of a unit: 8 floats, 16 bf16 or 16 floats
  };
  // A fragment of unit j (clamped like the B fragments): the patch values of this lane's site
  // for both 32-row blocks, and their low parts in split mode; unused members cost nothing
  auto a_load = [&](int j) {
    AFrag f;
    const float* ap = &s_mem[a_off(min(j, last))];
    f.h0 = *(const float4*)ap;
    f.h1 = (MB == 2 || NB == 16) ? *(const float4*)(ap + a_blk1) : f.h0;
    f.l0 = SPLIT ? *(const float4*)(ap + LO) : f.h0;
    f.l1 = (SPLIT && MB == 2) ? *(const float4*)(ap + a_blk1 + LO) : f.h0;
    return f;
  };
  auto unit = [&](const AFrag& af, const BFrag& bf) {
    const float4& b = bf.h;
    const float4 a0 = af.h0, a1 = af.h1;
    if (NB == 16) {
      c16a = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.x, b.x, c16a, 0, 0, 0);
      c16b = __builtin_amdgcn_mfma_f32_16x16x4f32(a1.x, b.x, c16b, 0, 0, 0);
      c16a = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.y, b.y, c16a, 0, 0, 0);
      c16b = __builtin_amdgcn_mfma_f32_16x16x4f32(a1.y, b.y, c16b, 0, 0, 0);
      c16a = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.z, b.z, c16a, 0, 0, 0);
      c16b = __builtin_amdgcn_mfma_f32_16x16x4f32(a1.z, b.z, c16b, 0, 0, 0);
      c16a = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.w, b.w, c16a, 0, 0, 0);
      c16b = __builtin_amdgcn_mfma_f32_16x16x4f32(a1.w, b.w, c16b, 0, 0, 0);
      return;
    }
    if (SPLIT) {
      // a * b ~ a_lo * b_hi + a_hi * b_lo + a_hi * b_hi (the low x low term, 2^-16 smaller, is dropped)
      const bf16x8 bh = __builtin_bit_cast(bf16x8, bf.h), bl = __builtin_bit_cast(bf16x8, bf.l);
      const bf16x8 a0h = __builtin_bit_cast(bf16x8, a0);
      const bf16x8 a0l = __builtin_bit_cast(bf16x8, af.l0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0l, bh, acc0, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0h, bl, acc0, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0h, bh, acc0, 0, 0, 0);
      if (MB == 2) {
        const bf16x8 a1h = __builtin_bit_cast(bf16x8, a1);
        const bf16x8 a1l = __builtin_bit_cast(bf16x8, af.l1);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1l, bh, acc1, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1h, bl, acc1, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1h, bh, acc1, 0, 0, 0);
      }
      return;
    }
    if (BF16) {
      const bf16x8 bb = __builtin_bit_cast(bf16x8, b);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a0), bb, acc0, 0, 0, 0);
      if (MB == 2) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a1), bb, acc1, 0, 0, 0);
      return;
    }
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.x, b.x, acc0, 0, 0, 0);
    if (MB == 2) acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.x, b.x, acc1, 0, 0, 0);
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.y, b.y, acc0, 0, 0, 0);
    if (MB == 2) acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.y, b.y, acc1, 0, 0, 0);
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.z, b.z, acc0, 0, 0, 0);
    if (MB == 2) acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.z, b.z, acc1, 0, 0, 0);
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.w, b.w, acc0, 0, 0, 0);
    if (MB == 2) acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.w, b.w, acc1, 0, 0, 0);
  };

  // Ring of three weight fragments, two units of look-ahead, no register copies: vector loads
  // complete in order, so each wait only covers loads issued two units earlier.  The first two
  // fragments of a chunk are requested before the barriers that precede it.
  BFrag bq0, bq1, bq2;
  bq0.h = bq0.l = make_float4(0.f, 0.f, 0.f, 0.f);
  bq1 = bq0;
  bq2 = bq0;
  EVK_PHASE(kPhAddressed);
  if (conv_on) {
    fetch(0);
    if (n_mine > 0) {
      bq0 = b_load(0, 0);
      bq1 = b_load(0, 1);
    }
  }
  EVK_PHASE(kPhFirstIssued);
#ifdef EVCONV_PHASE_STAMPS
  unsigned long long ph_contract = 0, ph_change = 0;
#endif
  for (int c0 = 0; conv_on && c0 < Cin; c0 += CHUNK) {
#ifdef EVCONV_PHASE_STAMPS
    const unsigned long long ph_a = wall_clock64();
#endif
    __syncthreads();  // all waves are done reading the previous chunk
    stash(c0);
    __syncthreads();
    if (ups) {
      interpolate();
      __syncthreads();
    }
    const bool more = c0 + CHUNK < Cin;
    if (more) fetch(c0 + CHUNK);  // next chunk's patch, in flight during the contraction
#ifdef EVCONV_PHASE_STAMPS
    const unsigned long long ph_b = wall_clock64();
    ph_change += ph_b - ph_a;
    if (c0 == 0) EVK_PHASE(kPhFirstPatchInLds);
#endif
    if (n_mine <= 0) continue;    // more waves than units (1 x 1 taps): only help with the gather
    // fp32 and bf16 modes: the A fragments run one unit ahead of their use (three names, two alive
    // at a time), so that an LDS read is in flight during the matrix instructions of the unit
    // before it.  Split mode has no registers to spare for that and reads each fragment at its use.
    constexpr bool APIPE = !SPLIT;
    int j = 0;
    AFrag aq0 = a_load(0), aq1 = aq0, aq2 = aq0;
    auto step = [&](AFrag& cur, AFrag& nxt, int jj, const BFrag& b) {
      if (APIPE) nxt = a_load(jj + 1); else cur = a_load(jj);
      unit(cur, b);
    };
    for (; j + 3 <= n_mine; j += 3) {
      bq2 = b_load(c0, j + 2);
      step(aq0, aq1, j, bq0);
      bq0 = b_load(c0, j + 3);
      step(aq1, aq2, j + 1, bq1);
      bq1 = b_load(c0, j + 4);
      step(aq2, aq0, j + 2, bq2);
    }
    if (j < n_mine) step(aq0, aq1, j, bq0);
    if (j + 1 < n_mine) step(aq1, aq2, j + 1, bq1);
    if (more) {
      bq0 = b_load(c0 + CHUNK, 0);
      bq1 = b_load(c0 + CHUNK, 1);
    }
#ifdef EVCONV_PHASE_STAMPS
    ph_contract += wall_clock64() - ph_b;
#endif
  }
  EVK_PHASE(kPhChunksDone);
#ifdef EVCONV_PHASE_STAMPS
  if (tid == 0 && ph_slot < kPhaseRecords) {
    g_phase[ph_slot][kPhContractionTicks] = ph_contract;
    g_phase[ph_slot][kPhChunkChangeTicks] = ph_change;
  }
#endif

  // operands of the fused ADD stages, requested together now so that one memory latency covers
  // all of them and the reduction below hides part of it
  float f_skip[kMaxFusedAdds][EP_ITERS], f_zold[kMaxFusedAdds][EP_ITERS];
#pragma unroll
  for (int f = 0; f < kMaxFusedAdds; ++f) {
#pragma unroll
    for (int it = 0; it < EP_ITERS; ++it) f_skip[f][it] = f_zold[f][it] = 0.0f;
    if (f >= p.n_fused) continue;
    const uint64_t skip_mine = mine(skip_word[f]);
    const __amdgpu_buffer_rsrc_t skip_rsrc = out_rsrc(at_stream(p.fused[f].skip, so));
#pragma unroll
    for (int it = 0; it < EP_ITERS; ++it) f_skip[f][it] = ep_load(skip_rsrc, has(skip_mine, it), it);
    if (p.fused[f].keeps_z && !p.dense) {
      const __amdgpu_buffer_rsrc_t fz_rsrc = out_rsrc(at_stream(p.fused[f].z, so));
#pragma unroll
      for (int it = 0; it < EP_ITERS; ++it) f_zold[f][it] = ep_load(fz_rsrc, has(site_mine, it), it);
    }
  }

  // residuals and rounding step of a fused sparsification layer
  float sp_delta[EP_ITERS];
  float sp_k = 0.0f;
#pragma unroll
  for (int it = 0; it < EP_ITERS; ++it) sp_delta[it] = 0.0f;
  if (p.sp.delta && !p.dense) {
    sp_k = *at_stream(p.sp.step, so);
    const __amdgpu_buffer_rsrc_t d_rsrc = out_rsrc(at_stream(p.sp.delta, so));
#pragma unroll
    for (int it = 0; it < EP_ITERS; ++it) sp_delta[it] = ep_load(d_rsrc, sp_k > 0.0f && has(site_mine, it), it);
  }

  EVK_PHASE(kPhFusedRequested);
  // ---- reduce the NW partial sums through LDS: slots [4][block*16 + reg][lane]
  auto spill = [&](float* part) {
    if (NB == 16) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        part[i * 64 + lane] = c16a[i];
        part[(4 + i) * 64 + lane] = c16b[i];
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      part[i * 64 + lane] = acc0[i];
      if (MB == 2) part[(16 + i) * 64 + lane] = acc1[i];
    }
  };
  __syncthreads();
  if (NW == 8) {
    if (wave >= 4) spill(s_mem + (wave - 4) * SLOT);
    __syncthreads();
    if (wave < 4) {
      const float* part = s_mem + wave * SLOT;
      if (NB == 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          c16a[i] += part[i * 64 + lane];
          c16b[i] += part[(4 + i) * 64 + lane];
        }
      }
#pragma unroll
      for (int i = 0; i < (NB == 16 ? 0 : 16); ++i) {
        acc0[i] += part[i * 64 + lane];
        if (MB == 2) acc1[i] += part[(16 + i) * 64 + lane];
      }
    }
  }
  if (wave < 4) spill(s_mem + wave * SLOT);
  __syncthreads();
  EVK_PHASE(kPhReduced);
#ifdef EVCONV_PHASE_STAMPS
  __builtin_amdgcn_s_waitcnt(0);  // (separates waiting for the operands from the epilogue's own time)
  EVK_PHASE(kPhArrived);
#endif

  // epilogue: thread -> (output channel = tid % 32, EP_ITERS sites); accumulator element
  // (block b, register i, lane l) is local site b*32 + 8*(i/4) + 4*(l/32) + i%4, channel l%32
  // (nonzero bits are collected where the thread's sites are, EP_SITES bits apart, and shifted to
  // their place in the tile word once)
  uint64_t nz_mine = 0;
  uint64_t nz_fused_mine[kMaxFusedAdds] = {0, 0};
  uint64_t nz_sp_mine = 0;
  const __amdgpu_buffer_rsrc_t o_rsrc = out_rsrc(at_stream(p.out, so));
  // partial sum of local site ls = it * EP_SITES + es: the part of the LDS offset that depends on
  // the thread (es < 16), the rest is a constant per `it`
  // (NB == 16: element (block b, register i, lane l) is local site 16 b + 4 (l / 16) + i, channel l % 16)
  const int off_mine = NB == 16 ? ((es >> 4) * 4 + (es & 3)) * 64 + ((es >> 2) & 3) * 16 + co
                                : ((es >> 3) * 4 + (es & 3)) * 64 + ((es >> 2) & 1) * 32 + co;
  const float bias = (p.dense && p.bias && co_ok) ? p.bias[co0 + co] : 0.0f;
  // Straight-line code: a site this thread does not own gets an out-of-range offset (its stores
  // are dropped) instead of a branch around it, and the partial sums of all passes are read from
  // LDS up front, so that the passes are not a chain of LDS round trips.
  float v_sum[EP_ITERS];
#pragma unroll
  for (int it = 0; it < EP_ITERS; ++it) {
    constexpr int kRow = EP_SITES / 8;  // tile rows per `it`
    const int off = NB == 16 ? off_mine + it * (EP_SITES / 16) * 4 * 64
                             : off_mine + (((it * kRow) >> 2) * 16 + ((it * kRow) & 3) * 4) * 64;
    v_sum[it] = (s_mem[off] + s_mem[off + SLOT]) + (s_mem[off + 2 * SLOT] + s_mem[off + 3 * SLOT]);
  }
  auto ep_store_at = [&](const __amdgpu_buffer_rsrc_t& r, unsigned voff, int it, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, voff, it * ep_step, 0);
  };
  // Activations other than none / ReLU need branches (exp, tanh); nets made of the two simple
  // ones, the usual case, take a loop without any: every decision that is the same for the whole
  // workgroup becomes a select, so that the passes can be interleaved freely (a branch per
  // decision and pass made each pass a chain of kernel-argument loads and waits).
  bool simple_acts = p.act == kActNone || p.act == kActRelu;
#pragma unroll
  for (int f = 0; f < kMaxFusedAdds; ++f)
    if (f < p.n_fused && p.fused[f].keeps_z && !(p.fused[f].act == kActNone || p.fused[f].act == kActRelu))
      simple_acts = false;
  auto epilogue_simple = [&](auto sp_tag) {
    constexpr bool HAS_SP = decltype(sp_tag)::value;
    const bool dense = p.dense != 0;
    const bool relu0 = p.act == kActRelu;
    bool f_on[kMaxFusedAdds], f_kz[kMaxFusedAdds], f_relu[kMaxFusedAdds];
    __amdgpu_buffer_rsrc_t f_out_r[kMaxFusedAdds], f_z_r[kMaxFusedAdds];
#pragma unroll
    for (int f = 0; f < kMaxFusedAdds; ++f) {
      f_on[f] = f < p.n_fused;
      f_kz[f] = f_on[f] && p.fused[f].keeps_z;
      f_relu[f] = f_kz[f] && p.fused[f].act == kActRelu;
      // (a stage that does not exist stores nowhere: its offsets are out of range)
      f_out_r[f] = out_rsrc(at_stream(f_on[f] ? p.fused[f].out : p.out, so));
      f_z_r[f] = out_rsrc(at_stream(f_kz[f] ? p.fused[f].z : p.out, so));
    }
    const __amdgpu_buffer_rsrc_t sp_delta_r = out_rsrc(at_stream(HAS_SP ? p.sp.delta : p.out, so));
    const __amdgpu_buffer_rsrc_t sp_out_r = out_rsrc(at_stream(HAS_SP ? p.sp.out : p.out, so));
#pragma unroll
    for (int it = 0; it < EP_ITERS; ++it) {
      const bool on_site = has(site_mine, it), on_conv = has(touched_mine, it);
      const unsigned at_site = on_site ? ep_voff : kSkipAccess, at_conv = on_conv ? ep_voff : kSkipAccess;
      // regular pass: z = v + bias, o = act(z); incremental: z += v, o = act(z_new) - act(z_old)
      // (z_old reads as 0 in a regular pass, so ReLU's difference form serves both)
      const float v = v_sum[it];
      const float z_new = (dense ? bias : z_old[it]) + v;
      ep_store_at(z_rsrc, at_conv, it, z_new);
      float o = relu0 ? fmaxf(z_new, 0.0f) - fmaxf(z_old[it], 0.0f) : (dense ? z_new : v);
      o = on_conv ? o : 0.0f;
      ep_store_at(o_rsrc, at_conv, it, o);
      if (o != 0.0f) nz_mine |= 1ull << (it * EP_SITES);
      // fused ADD nodes (Eq.11 followed by Eq.12-14): a = the value just produced, b = skip input
#pragma unroll
      for (int f = 0; f < kMaxFusedAdds; ++f) {
        const float lin = o + f_skip[f][it];
        const float z2_new = dense ? lin : f_zold[f][it] + lin;
        ep_store_at(f_z_r[f], f_kz[f] ? at_site : kSkipAccess, it, z2_new);
        float o2 = f_relu[f] ? fmaxf(z2_new, 0.0f) - fmaxf(f_zold[f][it], 0.0f) : lin;
        o2 = on_site ? o2 : 0.0f;
        ep_store_at(f_out_r[f], f_on[f] ? at_site : kSkipAccess, it, o2);
        if (f_on[f] && o2 != 0.0f) nz_fused_mine[f] |= 1ull << (it * EP_SITES);
        o = f_on[f] ? o2 : o;
      }
      // fused sparsification layer on the last stage's increment (Eq.3-8): x_corr = delta + x_inc,
      // y_inc = k floor(0.5 + x_corr / k), delta = x_corr - y_inc where x_inc is nonzero; elsewhere
      // y_inc = 0 and the residual stays.  A regular pass: identity, residual cleared.
      if (HAS_SP) {
#pragma clang fp contract(off)  // the residual is x_corr minus the rounded product, not a fused form
        const bool sp_on = sp_k > 0.0f, moved = o != 0.0f;   // (sp_k is 0 in a regular pass)
        const float x_corr = sp_delta[it] + o;
        const float q = sp_k * floorf(0.5f + x_corr / sp_k);
        const float y = sp_on ? (moved ? q : 0.0f) : o;
        ep_store_at(sp_delta_r, (dense || (sp_on && moved)) ? at_site : kSkipAccess, it, dense ? 0.0f : x_corr - y);
        ep_store_at(sp_out_r, at_site, it, y);
        if (y != 0.0f) nz_sp_mine |= 1ull << (it * EP_SITES);
      }
    }
  };
  if (simple_acts) {
    if (p.sp.delta) epilogue_simple(std::true_type{}); else epilogue_simple(std::false_type{});
  } else {
#pragma unroll
  for (int it = 0; it < EP_ITERS; ++it) {
    const bool on_site = has(site_mine, it), on_conv = has(touched_mine, it);
    const unsigned at_site = on_site ? ep_voff : kSkipAccess, at_conv = on_conv ? ep_voff : kSkipAccess;
    float o;
    {
      const float v = v_sum[it];
      if (p.dense) {
        const float z = v + bias;
        ep_store_at(z_rsrc, at_conv, it, z);
        o = act_m(p.act, z);
      } else {
        const float z_new = z_old[it] + v;
        ep_store_at(z_rsrc, at_conv, it, z_new);
        o = (p.act == kActNone) ? v : act_m(p.act, z_new) - act_m(p.act, z_old[it]);
      }
      o = on_conv ? o : 0.0f;
      ep_store_at(o_rsrc, at_conv, it, o);
      if (o != 0.0f) nz_mine |= 1ull << (it * EP_SITES);
    }
    // fused ADD nodes (Eq.11 followed by Eq.12-14): a = the value just produced, b = skip input
#pragma unroll
    for (int f = 0; f < kMaxFusedAdds; ++f) {
      if (f >= p.n_fused) break;
      const FusedAdd& fa = p.fused[f];
      const float lin = o + f_skip[f][it];
      if (fa.keeps_z) {
        const __amdgpu_buffer_rsrc_t fz_rsrc = out_rsrc(at_stream(fa.z, so));
        if (p.dense) {
          ep_store_at(fz_rsrc, at_site, it, lin);
          o = act_m(fa.act, lin);
        } else {
          const float z2_old = f_zold[f][it];
          const float z2_new = z2_old + lin;
          ep_store_at(fz_rsrc, at_site, it, z2_new);
          o = (fa.act == kActNone) ? lin : act_m(fa.act, z2_new) - act_m(fa.act, z2_old);
        }
      } else {
        o = lin;
      }
      o = on_site ? o : 0.0f;
      ep_store_at(out_rsrc(at_stream(fa.out, so)), at_site, it, o);
      if (o != 0.0f) nz_fused_mine[f] |= 1ull << (it * EP_SITES);
    }
    // fused sparsification layer on the last stage's increment (Eq.3-8): x_corr = delta + x_inc,
    // y_inc = k floor(0.5 + x_corr / k), delta = x_corr - y_inc where x_inc is nonzero; elsewhere
    // y_inc = 0 and the residual stays.  A regular pass: identity, residual cleared.
    if (p.sp.delta) {
#pragma clang fp contract(off)  // the residual is x_corr minus the rounded product, not a fused form
      float y = o;
      if (p.dense) {
        ep_store_at(out_rsrc(at_stream(p.sp.delta, so)), at_site, it, 0.0f);
      } else if (sp_k > 0.0f) {
        const float x_corr = sp_delta[it] + o;
        y = (o != 0.0f) ? sp_k * floorf(0.5f + x_corr / sp_k) : 0.0f;
        ep_store_at(out_rsrc(at_stream(p.sp.delta, so)), (o != 0.0f) ? at_site : kSkipAccess, it, x_corr - y);
      }
      ep_store_at(out_rsrc(at_stream(p.sp.out, so)), at_site, it, y);
      if (y != 0.0f) nz_sp_mine |= 1ull << (it * EP_SITES);
    }
  }
  }
  EVK_PHASE(kPhEpilogueDone);
  // A site is nonzero where one of its 32 channels is: lanes 0-31 of a wave hold site es = 2 * wave
  // of every pass, lanes 32-63 site 2 * wave + 1, so one ballot per pass gives the wave's two site
  // bits; the waves' words meet in LDS (no atomics: 64 lanes hitting one LDS word are served one
  // after the other, about 2 us per instruction).
  auto lds_or = [&](int slot, uint64_t mine_bits) {
    uint64_t w = 0;
#pragma unroll
    for (int it = 0; it < EP_ITERS; ++it) {
      const uint64_t b = __ballot(((mine_bits >> (it * EP_SITES)) & 1ull) != 0);
      if (NB == 16)  // four sites of 16 lanes each
        w |= (uint64_t)(((b & 0xffffull) ? 1u : 0u) | ((b & 0xffff0000ull) ? 2u : 0u) | ((b & 0xffff00000000ull) ? 4u : 0u) |
                        ((b >> 48) ? 8u : 0u)) << (it * EP_SITES);
      else
        w |= (uint64_t)(((unsigned)b != 0 ? 1u : 0u) | ((unsigned)(b >> 32) != 0 ? 2u : 0u)) << (it * EP_SITES);
    }
    if (lane == 0) s_nz[slot * NW + wave] = w << (r0 * 8 + (64 / NB) * wave);
  };
  auto nz_word = [&](int slot) {
    uint64_t w = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) w |= s_nz[slot * NW + i];
    return w;
  };
  EVK_PHASE(kPhFlagsBallot);
  lds_or(0, nz_mine);
#pragma unroll
  for (int f = 0; f < kMaxFusedAdds; ++f)
    if (f < p.n_fused) lds_or(1 + f, nz_fused_mine[f]);
  if (p.sp.delta) lds_or(1 + kMaxFusedAdds, nz_sp_mine);
  EVK_PHASE(kPhFlagsInLds);
  __syncthreads();
  EVK_PHASE(kPhFlagsBarrier);
  if (tid < 4 * (4 + 2 * kMaxFusedAdds)) {
    // Site bits of this workgroup into the words of up to 4 + 2 * (fused ADDs) sets: S and T of the
    // conv, then T and S of each fused ADD (Eq.11b), then T and S of a fused sparsification layer
    // (its T is the active set of the stage it reads).  All words of those sets are pre-zeroed and
    // the other workgroups of a tile OR their share in.  Four lanes per set: a weight-folded
    // workgroup's bits go to the words of the four up-sampled tiles over its stored tile, where
    // site (y, x) is bit (2 * (y % 4) + fpy, 2 * (x % 4) + fpx) of tile (y / 4, x / 4), one of them
    // per lane; otherwise the first of the four lanes writes the tile's own word.
    const int set = tid >> 2, part = tid & 3;
    // S of the producer as seen by this workgroup's rows and channels
    uint64_t s_prev = p.dense ? touched_word : nz_word(0);
    uint64_t bits = set == 0 ? s_prev : (set == 1 && wg_co == 0) ? touched_word : 0ull;
    uint64_t* words = set == 0 ? p.occ_out : set == 1 ? p.occ_touched : nullptr;
#pragma unroll
    for (int f = 0; f < kMaxFusedAdds; ++f) {
      if (f >= p.n_fused) break;
      const FusedAdd& fa = p.fused[f];
      const uint64_t t_f = s_prev | skip_word[f];  // Eq.11b
      const uint64_t nz_f = nz_word(1 + f);
      const uint64_t s_f = (fa.structural || p.dense) ? t_f : nz_f;
      if (set == 2 + 2 * f) { bits = t_f; words = fa.occ_touched; }
      if (set == 3 + 2 * f) { bits = s_f; words = fa.occ_out; }
      s_prev = s_f;
    }
    if (p.sp.delta) {
      const uint64_t nz_sp = nz_word(1 + kMaxFusedAdds);
      if (set == 2 + 2 * kMaxFusedAdds) { bits = s_prev; words = p.sp.occ_touched; }
      if (set == 3 + 2 * kMaxFusedAdds) { bits = p.dense ? s_prev : nz_sp; words = p.sp.occ_out; }
    }
    if (bits && words) {
      words = at_stream(words, so);
      if (!fold) {
        if (part == 0) atomicOr((unsigned long long*)&words[tile], (unsigned long long)bits);
      } else {
        const int a = part >> 1, b = part & 1;
        uint64_t spread = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const unsigned nib = (unsigned)(bits >> ((4 * a + r) * 8 + 4 * b)) & 0xfu;
          const unsigned wide = (nib & 1u) | ((nib & 2u) << 1) | ((nib & 4u) << 2) | ((nib & 8u) << 3);
          spread |= (uint64_t)wide << ((2 * r + fpy) * 8 + fpx);
        }
        if (spread)
          atomicOr((unsigned long long*)&words[(2 * tile_y + a) * p.go.tx + 2 * tile_x + b], (unsigned long long)spread);
      }
    }
  }
  EVK_PHASE(kPhEnd);
}

inline int chunk_for(const ConvParams& p) {
  // low-resolution layers (few workgroups, always 8 waves): 128-channel chunks halve the number of
  // gather round trips, which is what these latency-bound launches consist of
  if (p.stride == 1 && p.k <= 3 && p.gi.c % 128 == 0 &&
      (long long)p.go.tiles() * (p.c_out_pad / 32) * p.st.n * 2 < 512) return 128;
  if (p.stride == 1 && p.k <= 3 && p.gi.c % 64 == 0) return 64;
  if (p.stride == 1 && (p.gi.c % 32 == 0 || (p.gi.c % 16 != 0 && p.gi.c > 32))) return 32;  // ragged: fewer, padded chunks
  return 16;
}

template <int CHUNK, int NW, int OPM, int MB, int NB = 32>
void launch_variant(const ConvParams& p, hipStream_t s) {
  const int PH = (4 * MB - 1) * p.stride + p.k, PW = 7 * p.stride + p.k;
  // (rows of the patch are padded to a pitch of 32 modulo 64 words: at most 64 more per row)
  size_t lds = (size_t)PH * (PW * (OPM == kOpBf16 ? CHUNK / 2 + 4 : CHUNK + 4) + 64) * sizeof(float);
  const size_t part = (size_t)4 * MB * 16 * 64 * sizeof(float);  // partial sums reuse the patch
  // The operand that is read by every XCD in full should be the smaller one: the weights of the
  // high-resolution layers, the input of the low-resolution ones (k * k * c_out weights per input
  // channel against one value per stored site per input channel).  Measured on the 32 x 44 -> 64 x
  // 88 up-sampling conv (256 -> 128 channels, 5 x 5): 95 -> 86 us; neutral on the other layers.
  ConvParams q = p;
  const long long in_sites = p.upsample ? (long long)p.lo_h * p.lo_w : (long long)p.gi.h * p.gi.w;
  q.wg_swap = (long long)p.k * p.k * p.go.c > in_sites && p.go.tiles() * (2 / MB) <= 65535;
  dim3 grid(p.go.tiles() * (2 / MB), p.c_out_pad / NB, p.st.n);
  if (q.wg_swap) grid = dim3(p.c_out_pad / NB, p.go.tiles() * (2 / MB), p.st.n);
  if (CHUNK == 32 && p.upsample) {
    // the low-resolution source region behind the patch buffer
    lds += (size_t)(PH / 2 + 3) * (PW / 2 + 3) * (CHUNK + 4) * sizeof(float);
    if (lds < part) lds = part;
    hipLaunchKernelGGL((conv_mfma_kernel<CHUNK, NW, OPM, MB, CHUNK == 32>), grid, dim3(NW * 64), lds, s, q);
    return;
  }
  if (lds < part) lds = part;
  hipLaunchKernelGGL((conv_mfma_kernel<CHUNK, NW, OPM, MB, false, NB>), grid, dim3(NW * 64), lds, s, q);
}

// share of the chip's 256 CUs kept busy when n equally long workgroups run at once
inline double fill(long long n) { return (double)n / 256.0 / (double)((n + 255) / 256); }

template <int CHUNK, int OPM>
void launch_shape(const ConvParams& p, hipStream_t s) {
  const long long n2 = (long long)p.go.tiles() * (p.c_out_pad / 32) * p.st.n;  // workgroups with whole tiles
  // Whole tiles (two accumulators per wave, every weight fragment used twice) pay off only when
  // the launch fills the chip several times over and a workgroup has a long contraction; measured
  // on the layers of the evaluation networks, half tiles win everywhere else (more, shorter
  // workgroups: shorter prologues and patches, better balance)
  bool halves = !(n2 >= 512 && p.k * p.k * p.gi.c >= 1600) || fill(2 * n2) > fill(n2) + 0.1;
  const long long n = halves ? 2 * n2 : n2;
  bool eight = n < 512;  // few workgroups: 8 waves each split K further
  // fp32, few half-tile workgroups that fill the chip unevenly (384 on 256 CUs: half of the CUs get
  // two; 32 or 128: most CUs get none): blocks of 16 output channels instead of 32, twice the
  // workgroups at half the work.  Four waves each where that gives three workgroups per CU, eight
  // where the chip still is not full.  Measured: the 32 x 44 layers of the depth net 37 / 28 -> 32 /
  // 26 us, the 16 x 16 x 512 layers of the flow net 30 -> 23.5 us, ResNet-18's 7 x 7 x 512 layers
  // 29 -> 21 us.
  constexpr int kNarrowBlock = OPM == kOpF32 ? 16 : 32;
  if (OPM == kOpF32 && halves && eight && !p.upsample && fill(2 * n) > fill(n) + 0.1) {
    if (2 * n <= 256) launch_variant<CHUNK, 8, OPM, 1, kNarrowBlock>(p, s);
    else launch_variant<CHUNK, 4, OPM, 1, kNarrowBlock>(p, s);
    return;
  }
  if (CHUNK == 128) {  // chosen only for few workgroups: the 4-wave variants are not built
    if (halves) launch_variant<CHUNK, 8, OPM, 1>(p, s); else launch_variant<CHUNK, 8, OPM, 2>(p, s);
    return;
  }
  constexpr int NW4 = CHUNK == 128 ? 8 : 4;
  if (halves) {
    if (eight) launch_variant<CHUNK, 8, OPM, 1>(p, s); else launch_variant<CHUNK, NW4, OPM, 1>(p, s);
  } else {
    if (eight) launch_variant<CHUNK, 8, OPM, 2>(p, s); else launch_variant<CHUNK, NW4, OPM, 2>(p, s);
  }
}

template <int OPM>
void launch_any(const ConvParams& p, hipStream_t s) {
  switch (chunk_for(p)) {
    case 128: launch_shape<128, OPM>(p, s); break;
    case 64: launch_shape<64, OPM>(p, s); break;
    case 32: launch_shape<32, OPM>(p, s); break;
    default: launch_shape<16, OPM>(p, s); break;
  }
}

// Copies the phase records of this translation unit's kernels to `host` (32 x u64 each, at most
// max_records); returns how many workgroups have written one since the last reset, or -1 in a
// build without phase stamps.
inline int phase_stamps_read(unsigned long long* host, int max_records, bool reset) {
#ifdef EVCONV_PHASE_STAMPS
  unsigned n = 0;
  if (hipDeviceSynchronize() != hipSuccess) return -2;
  if (hipMemcpyFromSymbol(&n, HIP_SYMBOL(g_phase_n), sizeof(n)) != hipSuccess) return -2;
  const unsigned take = std::min(std::min(n, kPhaseRecords), (unsigned)std::max(max_records, 0));
  if (host && take && hipMemcpyFromSymbol(host, HIP_SYMBOL(g_phase), sizeof(unsigned long long) * 32 * take) != hipSuccess) return -2;
  if (reset) {
    const unsigned zero = 0;
    if (hipMemcpyToSymbol(HIP_SYMBOL(g_phase_n), &zero, sizeof(zero)) != hipSuccess) return -2;
  }
  return (int)n;
#else
  (void)host; (void)max_records; (void)reset;
  return -1;
#endif
}

}  // namespace

}  // namespace evk
