// Internal interface between the host-side planner (evconv_api.hip) and the gfx950 kernels.
// Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace evk {

// Mask tile: 8 x 8 sites = 64 = one wavefront, so one ballot yields a tile's occupancy word.
constexpr int kTile = 8;

// Geometry of one H x W x C tensor and of its tile grid.
struct Geo {
  int h, w, c;
  int tx, ty;  // tiles per row / per column
  __host__ __device__ int sites() const { return h * w; }
  __host__ __device__ int tiles() const { return tx * ty; }
};
inline Geo make_geo(int c, int h, int w) {
  Geo g;
  g.h = h; g.w = w; g.c = c;
  g.tx = (w + kTile - 1) / kTile;
  g.ty = (h + kTile - 1) / kTile;
  return g;
}

enum Act { kActNone = 0, kActRelu = 1, kActSigmoid = 2, kActTanh = 3, kActOneMinus = 4 };

// Independent streams (cameras) that share the weights: every stream owns a copy of the whole
// state region; copy number blockIdx.z of any state pointer lies blockIdx.z * stride bytes
// further on.  Launchers put the number of streams into the grid's z dimension.
struct Streams {
  size_t stride;  // bytes between the copies of one state pointer
  int n;          // number of streams (grid z)
};
template <class T>
__device__ __forceinline__ T* at_stream(T* q, size_t off) {
  return q ? (T*)((uintptr_t)q + off) : nullptr;
}

// ---- increment builder (Eq.1 + mask) ---------------------------------------------------
enum BuilderMode { kBuildFrame = 0, kBuildIncrement = 1, kBuildReset = 2, kBuildIncrementDense = 3 };
struct BuilderParams {
  const float* in;    // C x H x W: frame x(n), increment, or x0
  float* x_prev;      // C x H x W cached previous frame
  float* dx;          // H x W x C increment (full frame in reset mode)
  uint64_t* occ;      // per-tile occupancy of the input increment
  uint64_t* clear;    // words to zero before the layers run (all nodes' occupancy), or null
  int n_clear;
  Geo g;
  int mode;
  Streams st;
  size_t in_stride;   // bytes between the streams' inputs (contiguous [n][C][H][W])
};
void launch_builder(const BuilderParams& p, hipStream_t s);

// ---- sparse incremental convolution (Eq.10 at touched tiles, fused Eq.12-14) ------------
// An ADD node folded into the epilogue of the conv that produces one of its inputs (residual
// add + activation, or skip add): y_lin = conv_out + skip, then the usual accumulate /
// activation-increment / mask logic of the ADD node, written to the ADD node's own buffers.
struct FusedAdd {
  const float* skip;        // increment of the other input (same geometry as the conv output)
  const uint64_t* occ_skip; // its occupancy words
  float* z;                 // accumulated tensor of the ADD node (null if it keeps none)
  float* out;               // its increment buffer
  uint64_t* occ_out;        // its S words (pre-zeroed; OR-ed in)
  uint64_t* occ_touched;    // its T words (pre-zeroed; OR-ed in)
  int act, keeps_z, structural;
};
constexpr int kMaxFusedAdds = 2;
// A sparsification layer (Eq.3-8) folded into the same epilogue: it reads the increment the last
// stage of the epilogue has just produced (the conv's, or the last fused ADD's), at the sites the
// workgroup visits, and writes its own buffers.  Its touched set is that stage's active set.
struct FusedSparsify {
  float* delta;             // its residual (accumulated tensor); null = no such layer
  float* out;               // its increment buffer (the value in a regular pass, where it is the identity)
  uint64_t* occ_out;        // its S words (pre-zeroed; OR-ed in)
  uint64_t* occ_touched;    // its T words (pre-zeroed; OR-ed in)
  const float* step;        // device scalar: the rounding step k (0 = identity)
};

struct ConvParams {
  const float* in;          // H x W x C increment of the input node (full values if dense)
  const uint64_t* occ_in;   // its occupancy words
  const void* w;            // re-laid weights [k*k][c_in][c_out_pad] (fp32 or bf16)
  const float* bias;        // fp32 [c_out] or null; used by the dense pass only
  float* z;                 // H x W x C accumulated pre-activation
  float* out;               // H x W x C output increment (value in dense mode)
  uint64_t* occ_out;        // S_out words (pre-zeroed; OR-ed in)
  uint64_t* occ_touched;    // T words
  Geo gi, go;
  int c_out_pad;
  int k, stride, pad, act;
  int dense;                // 1: regular forward pass (all sites, z overwritten with bias)
  int n_fused;              // matrix-core kernel only: ADD nodes applied in the epilogue, in order
  FusedAdd fused[kMaxFusedAdds];
  FusedSparsify sp;         // matrix-core kernel only: applied behind the last stage of the epilogue
  Streams st;               // w and bias are shared by all streams
  // matrix-core kernel only: the input is the bilinear x2 up-sampling of `in` (lo_h x lo_w stored
  // sites, occ_in their occupancy words); gi describes the up-sampled tensor
  int upsample, lo_h, lo_w;
  // up-sampling variant, optional (null = off): weight folding.  conv o bilinear x2 is, for each
  // output phase (row parity, column parity), a fold_k x fold_k stride-1 conv on the stored tensor
  // wherever the window stays clear of the clamped image border (Eq.9: both are linear).
  // fold_list has one entry per 8 x 8 tile of the output: v >= 0 = that up-sampled tile, run
  // through the interpolating gather; v < 0 = -(1 + 4 * stored_tile + 2 * row parity + column
  // parity): the 64 outputs of one phase over one 8 x 8 tile of stored sites.  w_fold: the four
  // phases' weight sets, each in the layout of w with fold_k x fold_k taps.  fold_base[parity]:
  // first row (column) of the window relative to the stored site.
  const int* fold_list; const void* w_fold; int fold_k; int fold_base[2];
  // matrix-core kernel only, set by its launcher: the grid's x dimension runs over the blocks of
  // 32 output channels and y over the tiles, instead of the other way round
  int wg_swap;
  // few-channel pointwise kernel only: the node is a network output and the kernel keeps the
  // public tensors itself (y += increment, dy = increment; C x H x W); null otherwise.
  // int_mode is one of kIntStep / kIntReset / kIntRecompute.
  float* y; float* dy; int int_mode;
};
void launch_conv_valu(const ConvParams& p, hipStream_t s);
// fp32 MFMA variant; requires c_in >= 9 and c_out >= 16 (c_out_pad = c_out rounded up to 32).  The re-laid weights
// of all matrix-core variants carry conv_mfma_padded_cin input channels (zero rows beyond c_in).
bool conv_mfma_f32_supported(const ConvParams& p);
int conv_mfma_padded_cin(const ConvParams& p);
bool conv_mfma_upsample_supported(const ConvParams& p);
void launch_conv_mfma_f32(const ConvParams& p, hipStream_t s);
// bf16 MFMA variant (increments rounded to bf16 in the gather, bf16 weights, fp32 accumulation)
bool conv_mfma_bf16_supported(const ConvParams& p);
void launch_conv_mfma_bf16(const ConvParams& p, hipStream_t s);
// fp32 operands contracted as bf16 high/low parts (three bf16 MFMAs per product)
bool conv_mfma_split_supported(const ConvParams& p);
void launch_conv_mfma_split(const ConvParams& p, hipStream_t s);
// phase records of the matrix-core kernels of one operand mode (conv_mfma_impl.h: PhaseField): copies
// at most max_records records of 32 x u64 to host, returns the number written since the last
// reset; -1 in a build without -DEVCONV_PHASE_STAMPS, -2 if a copy fails
int conv_mfma_f32_phase_stamps(unsigned long long* host, int max_records, bool reset);
int conv_mfma_bf16_phase_stamps(unsigned long long* host, int max_records, bool reset);
int conv_mfma_split_phase_stamps(unsigned long long* host, int max_records, bool reset);
// 1 x 1 taps with at most 8 output channels, or LINEAR on a 1 x 1 grid; weights [c_out][c_in] fp32
bool conv_pointwise_supported(const ConvParams& p);
// true if launch_conv_pointwise(p) runs the per-tile kernel, which can also keep an output node's
// public tensors (ConvParams::y, dy)
bool conv_pointwise_integrates(const ConvParams& p);
void launch_conv_pointwise(const ConvParams& p, hipStream_t s);
// narrow-input variant: taps * c_in <= 128, c_out >= 16; weights re-laid per MFMA lane:
// conv_narrow_weight_floats(c_out_pad) fp32 values, W[k = tap * c_in + ci][co] at
// conv_narrow_weight_index(k, co), zeros elsewhere
bool conv_narrow_supported(const ConvParams& p);
size_t conv_narrow_weight_floats(int c_out_pad);
size_t conv_narrow_weight_index(int k, int co);
void launch_conv_narrow(const ConvParams& p, hipStream_t s);

// ---- elementwise / structural increment operators ---------------------------------------
// kEwConcatUp: concat whose first operand is the bilinear x2 up-sampling of `a` (never stored):
// ga is the stored low-resolution geometry of a, gb and go are at the output resolution
enum EwOp { kEwAdd = 0, kEwAct, kEwConcat, kEwUp2x, kEwPoolAcc, kEwPoolMax, kEwSparsify, kEwMul, kEwConcatUp };
struct EwParams {
  int op, act, dense, keeps_z, structural;
  Geo ga, gb, go;
  const float* a; const uint64_t* occ_a;
  const float* b; const uint64_t* occ_b;
  float* z;                 // accumulated tensor (pool: cached window max; pool-acc: pooled input)
  float* z2;                // elementwise multiply: accumulated second factor (z: the first)
  float* out;
  uint64_t* occ_out; uint64_t* occ_touched;
  int k, stride, pad;       // pooling window
  const float* step;        // sparsification layer: device scalar, the rounding step k
  Streams st;
};
void launch_elementwise(const EwParams& p, hipStream_t s);

// ---- rounding step of a sparsification layer: k = tp * RMS(x), 8 significant bits ---------------
// Two fixed-order reduction stages (no floating-point atomics): `partial` holds kRmsBlocks floats.
constexpr int kRmsBlocks = 256;
void launch_rms_step(const float* x, size_t n, float tp, float* partial, float* step_out, Streams st, hipStream_t s);

// ---- global average pool -----------------------------------------------------------------
struct GapParams {
  const float* a; const uint64_t* occ_a; Geo ga;
  float* z; float* out; uint64_t* occ_out; uint64_t* occ_touched;
  int act, dense;
  Streams st;
};
void launch_gap(const GapParams& p, hipStream_t s);

// ---- output integration (Eq.2) -------------------------------------------------------------
enum IntegrateMode { kIntStep = 0, kIntReset = 1, kIntRecompute = 2 };
struct IntegrateParams {
  const float* delta;       // H x W x C node output (increment, or value in reset/recompute)
  const uint64_t* occ;      // S_out words
  float* y; float* dy;      // C x H x W
  Geo g; int mode;
  Streams st;
};
void launch_integrate(const IntegrateParams& p, hipStream_t s);

// ---- recurrent state: the previous step's output of a later node -----------------------------
struct DelayParams {
  const float* src_out;       // H x W x C: the delayed node's increment of the previous step, or its
                              // value if the previous pass was a regular forward pass
  const uint64_t* occ_saved;  // the delayed node's S_out words of the previous step
  float* z;                   // value emitted so far
  float* out;                 // this step's increment (value in a regular pass)
  uint64_t* occ_out; uint64_t* occ_touched;
  Geo g;
  int dense;                  // this pass is a regular forward pass
  int last_dense;             // the previous pass was one
  int zero_state;             // reset: the state before the first frame is zero
  Streams st;
};
void launch_delay(const DelayParams& p, hipStream_t s);
// dst[i] = src[i], n 64-bit words per stream
void launch_copy_u64(uint64_t* dst, const uint64_t* src, size_t n, Streams st, hipStream_t s);

// ---- ordered compaction of occupancy words into ascending site lists -------------------------
struct SetDesc {
  const uint64_t* occ; int32_t* idx; int32_t* count; uint64_t* bitmap;
  int h, w, tx, ty;
};
void launch_build_lists(const SetDesc* sets_dev, int n_sets, int max_ty, Streams st, hipStream_t s);

void launch_fill_u64(uint64_t* p, size_t n, uint64_t v, Streams st, hipStream_t s);

// timing probes of the chip (chip_probes.hip); number of values written, or < 0
constexpr int kChipProbeValues = 23;
constexpr size_t kChipProbeScratch = 1u << 20;
int chip_probes(void* scratch, size_t scratch_bytes, hipStream_t s, float* out, int n);

}  // namespace evk
