// Device-side interface of libhs: parameter blocks and launch functions of the HIP
// kernels behind the four per-frame stages (format conversion, recurrent conv-net
// inference, postprocess, overlay; paper Section III-A).  Host code fills a parameter
// block once per layer at application creation and launches it per frame.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hs {

typedef _Float16 f16;

// How to launch a kernel whose single argument is one of the parameter blocks below:
// hipLaunchKernel(func, grid, block, {&params}, shmem, stream), or the same as a graph node.
struct KernelDesc {
  const void* func;
  dim3 grid, block;
  unsigned shmem;
};

// ---- stage 1: bilinear resize (exact integer) + normalise + interleave ----------------
constexpr int kMaxBatch = 16;   // streams one launch can serve (blockIdx.y = stream)

struct ResizeParams {
  const uint8_t* src[kMaxBatch];   // per stream: frame, RGB bytes, row pitch src_pitch (x16)
  int batch;
  size_t dst_img_stride;           // halves between the streams' padded images
  size_t dst32_img_stride;         // floats between the streams' planar fp32 tensors
  size_t src_pitch;
  int wi, hi, wo, ho;
  f16* dst;             // padded 4-channel fp16 image: pixel (y+pad_t, x+pad_l), pitch dst_w px
  int dst_w, pad_l, pad_t;
  float* dst_f32;       // optional planar fp32 [3][ho][wo]
  const float* lut32;   // 256 entries
  const f16* lut16;     // 256 entries
  float rcp_dx, rcp_dy;         // 1/(2*wo), 1/(2*ho): division estimates
  uint32_t d_magic, d_shift;    // floor(n / (4*wo*ho)) = mulhi(n, d_magic) >> d_shift for n < 2^31
};
KernelDesc describe(const ResizeParams& p);

// ---- stage 2: implicit-GEMM convolution on fp16 MFMA ------------------------------------
// Activations are pixel-major ("NHWC"): element (y, x, c) at in[(y*win + x)*cin_pitch + c].
// The K axis is cut into chunks of KC contiguous halves; chunk q belongs to tap
// q / chunks_per_tap = (ky, kx) = (tap / kw, tap % kw) and starts at channel
// (q % chunks_per_tap) * KC of input pixel (stride*oy + ky - pad, stride*ox + kx - pad).
// Out-of-range pixels read as zero.  First layers (3 input channels) use a padded
// 4-channel image and "row taps": kw = 1, a chunk spans several adjacent pixels.
struct ConvParams {
  const f16* in;
  const f16* wt;        // packed [cout_pad][ktot], ktot = nchunks*KC, zero rows above cout
  const f16* wt_frag;   // variant 6: the same weights in MFMA fragment order,
                        // [cout_pad / 32][Cin chunk][tap][K-step of 16][lane][8 halves], lane r + 32 h
                        // holding k = 16 * step + 8 * h .. + 7 of channel 32 * group + r
  int hin, win, cin_pitch;
  int hout, wout, m;    // m = batch*hout*wout output pixels (images stacked along m)
  int batch, img_m;     // images per launch, pixels per image (hout*wout)
  int cout, cout_pad;   // cout_pad: multiple of the block's N tile
  int kc;               // 16, 32 or 64
  int depth;            // prefetch depth in chunks: 4, or 8 (kc == 64 only)
  int variant;          // 0: generic tile of 64 consecutive pixels (k_conv_mfma)
                        // 1, 2, 3: 3x3/1 layers with a shared input patch (k_conv3x3_halo),
                        //    needs cin % 64 == 0; spatial tile 8 x 8 (1) or 8 x 16 (2, 3);
                        //    3 keeps one patch buffer and three weight stages, so that three
                        //    workgroups fit a CU (grids well beyond two workgroups per CU)
                        // 4: 3x3/2 pad-1 layers the same way (8 x 8 tile, patch stored as four
                        //    parity planes), optionally with the block's 1x1/2 projection of
                        //    the same input fused in (wt2 != NULL)
                        // 5: a whole 64 -> 64 -> 64 channel block (two 3x3/1 convolutions, ReLU
                        //    between, shortcut from the input, ReLU) in one launch
                        //    (k_block64_fused): wt = first, wt2 = second convolution, res = in
                        // 6: 3x3/1 layers with >= 2 Cin chunks on grids of >= 1.5 workgroups per CU:
                        //    8 x 16 tile as variant 2, weights read as MFMA fragments straight
                        //    from wt_frag into registers, no weight tile in LDS (k_conv3x3_dira)
                        // 7: 3x3/2 layers (+ fused 1x1/2 projection) on such grids, weights from
                        //    wt_frag / wt2_frag, fp16 outputs with cout % 64 == 0 or split-K
                        //    partials, no residual (k_conv3x3s2_dira)
  int tiles_x;          // variant 1..5: spatial tiles per output row
  int ntaps, kw, chunks_per_tap, nchunks, ktot;
  int stride, pad;
  // split-K: blockIdx.z handles chunks [z*chunks_per_split, ...)
  int nsplit, chunks_per_split;
  int tiles_m, tiles_n; // 64x64 output tiles; the grid is 8 * tiles_per_xcd workgroups
  int tiles_per_wg;     // variant 1..4: consecutive spatial tiles one workgroup walks (>= 1);
                        // workgroups = ceil(tiles_m / tiles_per_wg) * tiles_n * nsplit
  int tiles_per_xcd;    // ceil(workgroups / 8)
  int n_block;          // variant 1..4: channel tiles per block of the tile order (divides tiles_n;
                        // 1: spatial tile fastest, tiles_n: channel tile fastest)
  int frag_ok;          // host planning hint: the layer may use the fragment-weight kernels
                        // (fp16 output of whole 64-channel tiles or split-K partials, no residual)
  int use_partial;      // 1: store fp32 partial sums for a reduction kernel, no epilogue here
  float* partial;       // [nsplit][m][cout_pad] fp32
  // fused epilogue (use_partial == 0)
  f16* out;             // out[m*out_pitch + n]
  int out_pitch;
  const f16* res;       // optional residual, res[m*res_pitch + n]
  int res_pitch;
  int relu;
  float* out_f32;       // if set: planar fp32 out_f32[n*m_total + m] instead of `out`
  // variant 4 only: fused 1x1 stride-2 projection of the same input (no residual, no ReLU)
  const f16* wt2;       // packed [cout_pad][cin], or NULL
  const f16* wt2_frag;  // variant 7: the projection in MFMA fragment order,
                        // [cout_pad / 32][Cin chunk][K-step of 16][lane][8 halves], or NULL
  f16* out2; int out2_pitch;
  float* partial2;      // [nsplit][m][cout_pad] fp32 when use_partial
};
KernelDesc describe(const ConvParams& p);

// Sum split-K partials in split order, add residual, ReLU, store fp16 (or planar fp32).
struct SplitKEpilogueParams {
  const float* partial; int nsplit; int m; int cout; int cout_pad;
  f16* out; int out_pitch; const f16* res; int res_pitch; int relu; float* out_f32; int img_m;
  // optional second tensor reduced in the same launch (fused projection): plain fp16 store
  const float* partial2; f16* out2; int out2_pitch;
};
KernelDesc describe(const SplitKEpilogueParams& p);

// ConvLSTM gate non-linearities and state update from the gate pre-activations, plus the 1x1
// head on the new h.  partial: [nsplit][m][4*hid], channels ordered i, f, g, o (hid each);
// hid must be 256.  c: fp32 [m][hid] updated in place; h: fp16 written to h_out[m*h_pitch + j];
// logits[(image*8 + k)*img_m + pixel] = sum_j w_head[k][j] * h[pixel][j] (fp16 weights).
struct LstmEpilogueParams {
  const float* partial; int nsplit; int m; int hid;
  float* c; f16* h_out; int h_pitch;
  const f16* w_head; float* logits; int img_m;
};
KernelDesc describe(const LstmEpilogueParams& p);

// Stem of the ResNet-style backbone: 7x7 stride-2 pad-3 convolution 3 -> 64, ReLU, 3x3 stride-2
// pad-1 max-pool, fused.  in: padded 4-channel fp16 images (pad 3 on the top and left, zeros),
// hin x win pixels each with win even; wt: the [64][224] matrix, k = (ky*8 + px)*4 + ch, zero where
// px == 7 or ch == 3, in MFMA fragment order: [channel half][ky][K-step of 16][lane][8 halves]; out: pooled pixel-major [batch][hp][wp][64].
struct StemPoolParams {
  const f16* in; const f16* wt; f16* out;
  int hin, win;          // padded image
  int hc, wc;            // convolution output
  int hp, wp;            // pooled output
  int batch;
  int tiles_x, tiles_y;  // tiles of 8 x 15 pooled pixels
  int tiles_per_xcd;     // ceil(batch * tiles_y * tiles_x / 8)
};
KernelDesc describe(const StemPoolParams& p);

// ---- stage 3: postprocess -----------------------------------------------------------------
struct PostRecord {           // written by the kernel into pinned host memory
  int32_t argmax_idx[8];
  float peak[8];
  uint8_t present[8];
};
struct PostParams {
  const float* logits; int n;    // [8][n]
  float theta;                   // logit threshold
  float* heat; uint8_t* mask;    // [8][n]
  PostRecord* rec;               // host-visible
  int batch;                     // images: logits/heat/mask are [batch][8][n], rec[batch]
  uint8_t* kmap;                 // [batch][n]: lowest channel with mask set, 0xff if none
  // anchors of the annotation layer: marks[(image*8 + k)*2 + {0,1}] = frame position (cx, cy) of
  // the centre of tool k's argmax cell, cx = -1 when the tool is absent; NULL: not wanted
  int* marks;
  int wm, hm, wf, hf;            // map (n == wm*hm) and frame size, for the anchors
};
KernelDesc describe(const PostParams& p);

// ---- stage 4: overlay ---------------------------------------------------------------------
constexpr int kMaxLayers = 4;   // networks whose results one overlay launch can draw
// What one network contributes to the picture: its channel map, colours and annotations.
struct OverlayLayer {
  const uint8_t* kmap; int wm, hm;   // [batch][hm][wm]: lowest set mask channel or 0xff
  float rcp_wm;                      // 1/wm: division estimate (needs wf*wm and hf*hm below 2^31)
  int a;                             // Q8 alpha, 0..256
  uint32_t pal[8];                   // R | G<<8 | B<<16
  // annotation layer: cross-hair and 'T'<k> label per present tool, opaque, in tool order
  const int* marks;                  // anchors written by the postprocess kernel, NULL: none
  int arm, half, scale;              // marker arm / half thickness, pixels per glyph cell
  float rcp_scale;                   // 1/scale
  uint64_t glyph[9];                 // bit (5*row + col) of glyph g, col 0 = leftmost
};
struct OverlayParams {
  const uint8_t* src[kMaxBatch]; uint8_t* dst[kMaxBatch];   // per stream
  int batch; size_t pitch; int wf, hf;
  float rcp_gpr, rcp_hf, rcp_wf;     // 1/ceil(wf/16), 1/hf, 1/wf (ceil(wf/16)*hf below 2^31)
  int n_layers;                      // layers drawn in order, each over the one before
  OverlayLayer layer[kMaxLayers];
};
KernelDesc describe(const OverlayParams& p);

// ---- scratch for callers that cannot allocate ---------------------------------------------
// A fixed device array inside the library (one copy per GPU, held until the process ends) that
// can stand in for the split-K scratch of an application's workspace.  Returns the array's
// device address ON THE CURRENT DEVICE and its size; the address is looked up once per device.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
hipError_t static_scratch_address(void** d_ptr, size_t* bytes);

// ---- helpers ------------------------------------------------------------------------------
void launch_fill_zero(void* d, size_t bytes, hipStream_t s);   // bytes multiple of 16
void launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s);   // bytes multiple of 16

}  // namespace hs
