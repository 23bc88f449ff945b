// Launch descriptors shared by the host planner/runtime and the gfx950 kernels.
// Everything here is plain data: the planner fills these at plan time, the runtime patches
// the external input/output pointers and launches.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace xenos {

enum { DT_F32 = 0, DT_BF16 = 1 };

// Bytes of one tile row consumed per reduction step of the dense-conv kernel (64 bf16 / 32 fp32 elements).
// The packed weight layout depends on it, so host and kernels share the constant.
constexpr int kRowBytes = 128;

// How the rows (m) of an implicit-GEMM tile enumerate conv-output pixels.  The enumeration IS the
// linked dataflow of Section 4.1 / Figure 4: the producer walks pixels in the order its linked
// consumer (the pooling) reads them.
enum {
  M_FLAT = 0,     // m = (n*OH + oh)*OW + ow: no pooling, output written pixel-major
  M_ZIGZAG = 1,   // m = 4*window + (dy*2+dx): 2x2/s2 pooling windows are 4 consecutive rows (Figure 4 zig-zag)
  M_PATCH = 2,    // tile = spatial patch of one image, staged on chip, then pooled (any k/s/pad/ceil)
  M_GAP = 3       // tile = (image, channel tile); loops over the whole map, global average in registers
};

enum { POOL_NONE = 0, POOL_MAX = 1, POOL_AVG = 2, POOL_GAP = 3 };

// Tile configurations of the dense-conv kernel (block = 256 threads = 4 wavefronts).
struct TileCfg { int bm, bn, wm, wn; };
static const TileCfg kTileCfgs[] = {
  {128, 128, 64, 64},
  {128, 64, 64, 32},
  {64, 64, 32, 32},
  {32, 128, 32, 32},
};
static const int kNumTileCfgs = 4;
// Configuration index of the halo-staged 3x3 kernel: 256 pixels x 128 or 64 channels, 512 threads, TH x TW spatial tile.
static const int kHaloCfg = 4;
// Configuration index of the first-layer kernel: 32 pixels x K (32 or 64) channels per wavefront, the reduction
// C*R*S (at most kStemRed, in up to kStemPasses MFMA passes of 32) gathered straight from the graph input through `ktab`.
static const int kStemCfg = 5;
static const int kStemPasses = 5;
static const int kStemRed = 32 * kStemPasses;
// Configuration index of the kernel that links the first two 3x3 convolutions (intermediate tensor kept in LDS): at most
// 4 input channels -> kPairChannels -> kPairChannels; the first convolution reduces over kPairRed slots = tap * 4 + channel.
static const int kPairCfg = 6;
// Configuration index of the kernel that streams the weights of a fully connected chain with at most 32 rows (128 channels per
// workgroup, reduction shared out over workgroups; always followed by the summing pass)
static const int kFcCfg = 7;
static const int kFcChannels = 128;
// Configuration index of the first-layer kernel that stages its input block in LDS (bf16 path, fp32 NCHW graph input with at most 4
// channels, square kernel up to 7x7, stride 1 or 2): tiles of kStemLdsTh x kStemLdsTw output pixels of one image
static const int kStemLdsCfg = 8;
static const int kStemLdsPph = 3, kStemLdsPpw = 8;   // pooling windows per tile when a max-pooling is linked
static const int kStemLdsTh = 8, kStemLdsTw = 16, kStemLdsInMax = 784;   // (7 * 2 + 7) x (15 * 2 + 7) = 777 positions at most
// (per kernel size class the kernel is instantiated for, by taps: up to 3x3 at stride 2 a block is at most 17 x 33 or 15 x 35
// positions, up to 5x5 19 x 35)
static inline int stem_lds_in_positions(int taps) { return taps <= 12 ? 576 : taps <= 28 ? 672 : kStemLdsInMax; }
// Configuration index of the kernel that links a pointwise (1x1) convolution chain with the depthwise 3x3 chain that consumes
// it: a TH x TW block of depthwise output pixels x kPwDwChannels channels per workgroup, the pointwise output of the block
// (+ halo) staged in LDS, at most kPwDwMaxPositions positions
static const int kPwDwCfg = 9;
static const int kPwDwChannels = 64, kPwDwMaxPositions = 400;
// Configuration index of the kernel that runs a Fire module (squeeze 1x1 -> expand 1x1 || expand 3x3 -> concat [-> max-pooling])
// as one chain: the squeeze output of a tile (+ halo, at most kFireMaxPositions positions, at most 64 channels) stays in LDS
static const int kFireCfg = 10;
static const int kFireMaxPositions = 400;
static const int kFcWgPerCu = 1;
static const int kFcDirectSteps = 16;   // reductions of at most this many 64-element steps are not shared out (no summing pass)    // workgroups per compute unit the reduction split of such a chain aims at
static const int kPairChannels = 64, kPairRed = 48;
static const int kPairRows = 128, kPairPatchMax = 180;   // output pixels and patch positions ((TH+2) x 18) of a tile
static const int kPairInMax = 256;   // positions of the staged block of the graph input, (TH+4) x (TW+4) plus slack for the pitch columns
static const int kHaloRows = 256, kHaloCols = 128, kHaloPatchMax = 360;
static const long long kL2BytesPerXcd = 4ll << 20;   // gfx950: one 4 MB L2 per XCD
// the staged patch has one of two fixed row pitches (pixels): tiles up to 16 or up to 32 pixels wide
static const int kHaloPitchTiny = 10, kHaloPitchNarrow = 18, kHaloPitchWide = 34;

struct ConvArgs {
  const void* in;        // activations: NHWC in the compute type (vector loader), or any strided fp32/T tensor (scalar loader)
  const void* w;         // packed weights [Kout_pad][Kred_pad] in the compute type, reduction index = (r*S+s)*C + c
  const float* scale;    // folded per-channel scale [Kout_pad] (1 where no BN)
  const float* shift;    // folded per-channel shift [Kout_pad]
  const void* res;       // residual (NHWC view, compute type) or nullptr
  const void* zeros;     // 256 bytes of zeros in device memory: what a masked 16-byte load reads (dwpw_kernel)
  void* out;
  const int32_t* ktab;   // scalar loader only: per reduction index {offset, (r<<16)|s}
  int N, C, H, W;
  long long in_sN, in_sH, in_sW;   // element strides of the input view (channel stride is 1 for the vector loader)
  int in_f32;            // scalar loader: input elements are fp32 (graph input) instead of the compute type
  int K, R, S, stride, pad, OH, OW;
  int Kred, Kred_pad;    // R*S*C and its padding to the reduction step
  int kchunk;            // reduction order: 1 = (channel chunk, r, s, channel in chunk), needs C % step == 0; 0 = (r, s, c)
  int mode;              // M_*
  int relu, has_res;
  // != 0: the chain also performs the two-group channel shuffle of the concat it ends in.  `res` is the other part of the
  // concat (strides res_sN / res_sP), `out` the concat buffer (2 K channels per pixel); channel k of this chain is stored
  // at output channel 2k + (ileave - 1) and channel k of the other part at 2k + (2 - ileave).  M_FLAT, general and
  // depthwise-panel kernels, 16-byte aligned channel groups only.
  int ileave;
  long long res_sN, res_sP;        // residual strides (image, pixel); channel stride 1
  int pool, pk, ps, pp, PH, PW, cip;   // linked pooling (POOL_*), window, stride, pad, pooled size, count_include_pad
  int patch_h, patch_w, pph, ppw, patches_y, patches_x;   // M_PATCH geometry (conv-output patch, pooled patch)
  long long out_sN, out_sP, out_sK;    // output strides (image, pixel, channel) in elements
  int out_f32;           // store fp32 instead of the compute type (graph output)
  int vec_out, vec_res;  // 16-byte channel-group stores / shortcut loads are legal (alignment, unit channel stride, K % group == 0)
  // linked depthwise producer (nullptr = none): `in` is then the depthwise INPUT (NHWC), H x W the depthwise output
  const void* dw_w; const float* dw_scale; const float* dw_shift;   // [k*k][C] compute type, folded scale / shift [C]
  int dw_k, dw_stride, dw_pad, dw_H, dw_W, dw_relu;
  long long dw_sN, dw_sP;
  // linked first-layer producer (pair kernel): `in` is the caller's fp32 NCHW tensor (unit stride along W) with pair_C
  // channels, dw_w its packed weights [kPairChannels][kPairRed], dw_scale / dw_shift / dw_relu its epilogue; C, H, W
  // describe the intermediate tensor
  int pair, pair_C;
  long long pair_sN, pair_sC, pair_sH;
  int dw_panel;          // > 0: the depthwise result of a whole panel of this many channels is staged in LDS (dwpw_kernel)
  // linked depthwise CONSUMER (pwdw_kernel): this 1x1 / stride 1 chain's output tile stays in LDS and a depthwise 3x3 chain
  // (dw_w [9][K], dw_scale / dw_shift [K], dw_stride, dw_pad = 1, dw_relu) runs out of it; H x W is the pointwise map,
  // OH x OW the depthwise output, th x tw the tile of depthwise output pixels, tiles_y x tiles_x the tile grid per image
  int pwdw;
  // linked Fire module (fire_kernel): this 1x1 / stride 1 chain is the squeeze (K <= 64 channels); its output tile (+ halo)
  // stays in LDS and two expand chains read it there: [0] 1x1, [1] 3x3 / pad 1.  fire_w: [E padded to 64][taps][K] in the
  // compute type; fire_scale / fire_shift: folded epilogue, padded to 64; fire_out: where each part goes (NHWC view of the
  // compute type: image stride fire_sN, pixel pitch fire_sP), after the linked max-pooling (pool, pk, ps, pp, PH, PW; tiles of
  // pph x ppw windows) if there is one; th x tw = tile of output pixels otherwise; tiles_n = channel shares
  int fire;
  const void* fire_w[2]; const float* fire_scale[2]; const float* fire_shift[2];
  void* fire_out[2]; long long fire_sN[2], fire_sP[2];
  int fire_E[2], fire_relu[2];
  // reduction split across workgroups (ksplit >= 1, M_FLAT only; 0 = none): share z covers steps [z*steps_per_split, ...)
  // and writes raw fp32 sums to part[z][m][k] (row pitch part_ld); a splitk_finish pass completes the chain
  int ksplit, steps_per_split, part_ld;
  float* part;
  int th, tw, tiles_y, tiles_x;   // halo kernel: spatial tile and tile grid over the stacked padded rows n*(H+2)+oh
  int halo_bn;           // halo kernel: output channels per tile (128 or 64)
  int halo_mgroup;       // halo kernel: an XCD walks its pixel tiles in groups of this many, every output-channel tile of a group
                         // before the next group (>= 1; a value of at least the XCD's tile count = one sweep per channel tile)
  int halo_plin;         // halo kernel: patch-linear rows (GEMM row = patch position, pitch TW + 2; pixel-major chains only)
  int M_total;           // rows enumerated over the whole problem (FLAT, ZIGZAG); per-image rows for GAP
  int tiles_m, tiles_n, ntiles;
  int xcd_m;             // dense-conv kernel: the 8 XCDs form an xcd_m x (8/xcd_m) grid over pixel tiles x (channel tiles x shares)
  int grid;              // workgroups launched (>= 1); tiles are visited with a stride of `grid`
};

struct DwArgs {
  const void* in; const void* w;     // w: [R*S][C] in the compute type
  const float* scale; const float* shift;
  void* out;
  int N, C, H, W, R, S, stride, pad, OH, OW;
  long long in_sN, in_sP;            // NHWC view strides (image, pixel)
  long long out_sN, out_sP;
  int relu;
  long long total_vec;               // N*OH*OW*(C/vec)
};

// Stand-alone passes of the un-linked baselines (and of whatever the link pass could not absorb).
enum { ELT_AFFINE = 0, ELT_RELU = 1, ELT_ADD = 2, ELT_COPY = 3 };
struct EltArgs {
  const void* a; const void* b; void* out;
  const float* scale; const float* shift;
  int op, relu;                      // relu applied after op when set
  int C;                             // channels of the view
  long long pixels;                  // N*H*W
  long long a_sP, b_sP, out_sP;      // pixel strides of the NHWC views
  long long a_sK, out_sK;            // channel strides of a and out (1 except for the strided copies of a channel shuffle)
};

struct PoolArgs {
  const void* in; void* out;
  int N, C, H, W, OH, OW, k, s, p, kind, cip;   // kind: POOL_MAX / POOL_AVG / POOL_GAP
  long long in_sN, in_sP, out_sN, out_sP;
};

// Layout / type conversion at the graph boundary (the transpose operator of Table 3).
struct CvtArgs {
  const void* in; void* out;
  int N, C, H, W;
  int Cout;                          // channels written per pixel (>= C; channels C..Cout-1 are zero-filled)
  long long in_sN, in_sC, in_sP;     // element strides: image, channel, pixel (pixel index = h*W + w)
  long long out_sN, out_sC, out_sP;
  int in_f32, out_f32;
};

struct SplitKArgs {
  const float* part; int ksplit, part_ld;
  int M, K, OHW;                     // rows (n*OH*OW), output channels, pixels per image
  const float* scale; const float* shift;
  const void* res; long long res_sN, res_sP;
  void* out; long long out_sN, out_sP, out_sK;
  int relu, out_f32;
  int gap;                           // 1: average the finished pixels of every image (linked global average), out = [image][K]
};

// Launchers (defined in xenos_kernels.hip).  dtype = DT_*.  Return a hipError_t value as int.
int launch_conv(const ConvArgs& a, int dtype, int cfg, int scalar_loader, void* stream);
int launch_dw(const DwArgs& a, int dtype, void* stream);
int launch_elt(const EltArgs& a, int dtype, void* stream);
int launch_pool(const PoolArgs& a, int dtype, void* stream);
int launch_cvt(const CvtArgs& a, int dtype, void* stream);
int launch_splitk_finish(const SplitKArgs& a, int dtype, void* stream);
size_t conv_lds_bytes(int cfg, int mode);
bool conv_cfg_has_scalar_loader(int cfg);
bool conv_cfg_has_dw_prologue(int cfg, int mode);
size_t dwpw_lds_bytes(int panel_channels, int esz);   // LDS of the depthwise-panel kernel for a panel of that many channels
// device probes for the roofline denominators (xenos_kernels.hip)
int launch_probe_mfma(void* d_out, int num_cu, int iters, int data, void* stream, double* flops);
int launch_probe_read(const void* d_in, size_t bytes, void* d_out, int num_cu, void* stream);
size_t probe_out_bytes(int num_cu);
// pointwise -> depthwise kernel (xenos_linked.hip)
int launch_pwdw(const ConvArgs& a, int dtype, void* stream);
size_t pwdw_lds_bytes(int th, int tw, int stride, int esz);
// Fire-module kernel (xenos_linked.hip); conv_h x conv_w = conv-output pixels of a tile
int launch_fire(const ConvArgs& a, int dtype, void* stream);
size_t fire_lds_bytes(int conv_h, int conv_w, int S, int esz, int pooled, int ring = 1);   // ring: halo of the block (1 with a 3x3 part)

}  // namespace xenos
