// HIP kernels (gfx950 / CDNA4 only) of the per-frame tool-tracking hot path:
// paper Section III-A stages format conversion -> inference -> postprocess -> overlay.
#include "hs_kernels.h"

#include <algorithm>
#include <mutex>

namespace hs {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // plain 16-byte register value

// floor(num / d) for num, d < 2^31 where the quotient is < 2^22: float estimate, exact fix-up.
__device__ __forceinline__ uint32_t udiv_est(uint32_t num, uint32_t d, float rcp_d) {
  uint32_t q = (uint32_t)((float)num * rcp_d);
  int32_t r = (int32_t)(num - q * d);
  if (r < 0) { q -= 1; r += (int32_t)d; }
  if (r >= (int32_t)d) { q += 1; }
  return q;
}

// =============================================================================================
// Stage 1: one workgroup per output row.  The two source rows the row needs are staged in
// LDS with 16-byte loads; every output pixel is the exact integer 4-tap sum, rounded once.
// =============================================================================================
// a * b (+ c) on the low 24 bits of a and b, low 32 bits of the result: the full-rate integer
// multiplier (the 32 x 32-bit one runs at a quarter of its rate).  Written as instructions
// because the compiler turns __umul24 back into a 32-bit multiply when it knows one factor
// to be small.
__device__ __forceinline__ uint32_t mul24(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_mul_u32_u24 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ uint32_t mad24(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Block size: 256..512 threads, chosen by the host so that the passes over the output row are as
// full as possible (854 pixels: two passes of 448 threads instead of four of 256) and that a
// source row is at most kResizeVecs 16-byte vectors per thread.  The row loads are the first
// thing a workgroup issues: the lookup tables and the row arithmetic are set up behind them.
constexpr int kResizeVecs = 4;
template <int NV>   // 16-byte vectors per thread and source row: 1, 2 or 4
__global__ __launch_bounds__(512) void k_resize_norm(ResizeParams p) {
  extern __shared__ __align__(16) uint8_t lds[];
  __shared__ float s_lut32[256];
  __shared__ f16 s_lut16[256];
  const int tid = threadIdx.x, T = blockDim.x;
  const int Y = blockIdx.x;
  const uint8_t* const src = p.src[blockIdx.y];          // stream blockIdx.y of the batch
  f16* const dst = p.dst + blockIdx.y * p.dst_img_stride;
  float* const dst_f32 = p.dst_f32 ? p.dst_f32 + blockIdx.y * p.dst32_img_stride : nullptr;
  const uint32_t dy = 2u * (uint32_t)p.ho, dx = 2u * (uint32_t)p.wo;
  int ny = (2 * Y + 1) * p.hi - p.ho;
  ny = max(0, min(ny, (p.hi - 1) * (int)dy));
  const uint32_t y0 = udiv_est((uint32_t)ny, dy, p.rcp_dy);
  const uint32_t fy = (uint32_t)ny - y0 * dy;
  const uint32_t y1 = min(y0 + 1u, (uint32_t)(p.hi - 1));

  // the two source rows: 16-byte loads into named registers (as arrays they end up in scratch
  // memory), addresses clamped to the row so that every load is unconditional
  const int row_vecs = (3 * p.wi + 15) >> 4;          // 16-byte vectors per source row
  const uint4* const row0 = reinterpret_cast<const uint4*>(src + (size_t)y0 * p.src_pitch);
  const uint4* const row1 = reinterpret_cast<const uint4*>(src + (size_t)y1 * p.src_pitch);
  uint4 st0_0, st0_1, st0_2, st0_3, st1_0, st1_1, st1_2, st1_3;
#define HS_FETCH_VEC(I_)                                                                       \
  if constexpr (NV > I_) {                                                                     \
    const int v_ = min(tid + I_ * T, row_vecs - 1);                                            \
    st0_##I_ = row0[v_];                                                                       \
    st1_##I_ = row1[v_];                                                                       \
  }
#define HS_HAND_VEC(I_)                                                                        \
  if constexpr (NV > I_) {                                                                     \
    if (tid + I_ * T < row_vecs) {                                                             \
      l0[tid + I_ * T] = st0_##I_;                                                             \
      l1[tid + I_ * T] = st1_##I_;                                                             \
    }                                                                                          \
  }
  HS_FETCH_VEC(0) HS_FETCH_VEC(1) HS_FETCH_VEC(2) HS_FETCH_VEC(3)
  if (tid < 256) {
    s_lut32[tid] = p.lut32[tid];
    s_lut16[tid] = p.lut16[tid];
  }
  uint4* const l0 = reinterpret_cast<uint4*>(lds);
  uint4* const l1 = l0 + row_vecs;
  const uint32_t* const p0 = reinterpret_cast<const uint32_t*>(lds);
  const uint32_t* const p1 = reinterpret_cast<const uint32_t*>(lds + (size_t)row_vecs * 16);
  const uint32_t d = dx * dy;

  HS_HAND_VEC(0) HS_HAND_VEC(1) HS_HAND_VEC(2) HS_HAND_VEC(3)
  __syncthreads();
  const uint32_t wy1 = fy, wy0 = dy - fy;
  for (int X = tid; X < p.wo; X += T) {
    int nx = (2 * X + 1) * p.wi - p.wo;
    nx = max(0, min(nx, (p.wi - 1) * (int)dx));
    const uint32_t x0 = udiv_est((uint32_t)nx, dx, p.rcp_dx);
    const uint32_t fx = (uint32_t)nx - x0 * dx;
    const uint32_t wx1 = fx, wx0 = dx - fx;
    // The two source pixels x0, x0+1 are 6 consecutive bytes inside three aligned words: fetch
    // the words from each row and funnel-shift the bytes into place (v_alignbyte).  At the
    // right edge x0 + 1 is past the row, its weight fx is 0 there and the bytes read are the
    // next row or the padding behind the rows.
    const uint32_t b0 = 3u * x0, wi0 = b0 >> 2, sh = b0 & 3u;
    const uint32_t a0 = __builtin_amdgcn_alignbyte(p0[wi0 + 1], p0[wi0], sh);      // bytes 0..3
    const uint32_t a1 = __builtin_amdgcn_alignbyte(p0[wi0 + 2], p0[wi0 + 1], sh);  // bytes 4..7
    const uint32_t c0 = __builtin_amdgcn_alignbyte(p1[wi0 + 1], p1[wi0], sh);
    const uint32_t c1 = __builtin_amdgcn_alignbyte(p1[wi0 + 2], p1[wi0 + 1], sh);
    const uint64_t r0 = (uint64_t)a1 << 32 | a0, r1 = (uint64_t)c1 << 32 | c0;
    uint32_t q[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      const uint32_t p00 = (uint32_t)(r0 >> (8 * c)) & 0xffu, p01 = (uint32_t)(r0 >> (8 * c + 24)) & 0xffu;
      const uint32_t p10 = (uint32_t)(r1 >> (8 * c)) & 0xffu, p11 = (uint32_t)(r1 >> (8 * c + 24)) & 0xffu;
      // every factor is below 2^24 (weights <= 2*wo, 2*ho <= 2^15; a row sum <= 2*wo*255 < 2^24) and
      // the sum below 2^31: 24-bit multiplies are exact here and run at four times the rate of
      // the 32-bit ones
      const uint32_t acc = mad24(wy0, mad24(wx0, p00, mul24(wx1, p01)),
                                 mul24(wy1, mad24(wx0, p10, mul24(wx1, p11))));
      // floor((acc + d/2) / d) by multiplication: exact for numerators below 2^31
      q[c] = __umulhi(acc + (d >> 1), p.d_magic) >> p.d_shift;
    }
    half4 px;
    px[0] = s_lut16[q[0]];
    px[1] = s_lut16[q[1]];
    px[2] = s_lut16[q[2]];
    px[3] = (f16)0.0f;
    *reinterpret_cast<half4*>(dst + ((size_t)(Y + p.pad_t) * p.dst_w + (X + p.pad_l)) * 4) = px;
    if (dst_f32) {
      const size_t plane = (size_t)p.ho * p.wo;
      float* o = dst_f32 + (size_t)Y * p.wo + X;
      o[0] = s_lut32[q[0]];
      o[plane] = s_lut32[q[1]];
      o[2 * plane] = s_lut32[q[2]];
    }
  }
#undef HS_HAND_VEC
#undef HS_FETCH_VEC
}

static unsigned resize_block(const ResizeParams& p) {
  const unsigned row_vecs = (unsigned)((3 * p.wi + 15) >> 4);
  const unsigned t_min = std::max(256u, (row_vecs + kResizeVecs - 1) / kResizeVecs);
  unsigned best = 0;
  for (unsigned t = 256; t <= 512; t += 64) {
    if (t < t_min) continue;
    if (!best || (p.wo + t - 1) / t * t < (p.wo + best - 1) / best * best) best = t;
  }
  return best ? best : 512;
}

KernelDesc describe(const ResizeParams& p) {
  const unsigned lds = (unsigned)((3 * p.wi + 15) >> 4) * 16 * 2 + 16;   // + padding read at the edge
  const unsigned t = resize_block(p);
  const unsigned nv = ((unsigned)((3 * p.wi + 15) >> 4) + t - 1) / t;
  const void* f = nv <= 1   ? (const void*)k_resize_norm<1>
                  : nv == 2 ? (const void*)k_resize_norm<2>
                            : (const void*)k_resize_norm<kResizeVecs>;
  return KernelDesc{f, dim3(p.ho, p.batch), dim3(t), lds};
}

// =============================================================================================
// Stage 2: implicit-GEMM convolution.  A workgroup (4 wavefronts) owns a 64-pixel x 64-channel
// output tile; each wavefront owns a 32x32 quarter and accumulates it with
// v_mfma_f32_32x32x16_f16.  The MFMA "A" operand is the weight tile and the "B" operand the
// pixel tile, so a lane ends up holding 4 consecutive output channels of one pixel per
// accumulator quad -> 8-byte fp16 stores into the pixel-major output.
//
// Latency hiding: at batch 1 a grid is only 1-2 workgroups per CU, so the K loop keeps DEPTH
// chunks of global loads in flight in registers (the loads of chunk q+DEPTH are issued right
// after chunk q has been handed to LDS); LDS is double buffered, one barrier per chunk.
//
// Split-K: blockIdx.z owns a contiguous range of chunks and stores fp32 partial sums; the
// reduction kernels below sum them in split order and run the epilogue.
// =============================================================================================
__device__ __forceinline__ float sigmoid_f(float x) { return 1.0f / (1.0f + __expf(-x)); }

// residual add, ReLU and store of 4 consecutive output channels n..n+3 of pixel m
template <bool LOAD_RES = true>
__device__ __forceinline__ void store_quad(const ConvParams& p, int m, int n, float v[4]) {
  if (LOAD_RES && p.res) {
    const half4 r = *reinterpret_cast<const half4*>(p.res + (size_t)m * p.res_pitch + n);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] += (float)r[j];
  }
  if (p.relu) {
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = fmaxf(v[j], 0.0f);
  }
  if (p.out_f32) {
    // planar per image: out_f32[(image * cout + channel) * img_m + pixel in image]
    const int b = m / p.img_m, ml = m - b * p.img_m;
#pragma unroll
    for (int j = 0; j < 4; ++j) p.out_f32[((size_t)b * p.cout + n + j) * p.img_m + ml] = v[j];
  } else {
    half4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (f16)v[j];
    *reinterpret_cast<half4*>(p.out + (size_t)m * p.out_pitch + n) = o;
  }
}

// Epilogue of the 32 channels of one pixel that a lane pair (r, r + 32) holds as accumulator
// quads: lane half h has channels cbase + 4h + 8i .. +3 in acc[4i .. 4i+3], i = 0..3.  Residual,
// ReLU and rounding to fp16 as in store_quad; then the two lanes swap one quad of every pair
// (v_permlane32_swap: lanes 32..63 of the first operand <-> lanes 0..31 of the second), so that
// each holds 8 consecutive channels per pair and stores 16 bytes at a time instead of 8.
// For fp16 outputs whose channel count is a multiple of 32.  Every lane of the wavefront must
// call it (the swap needs both lanes of a pair); `valid` gates the store.  out / pitch / relu:
// the destination tensor (the layer's output, or the projection's).
__device__ __forceinline__ void store_octets_to(f16* out, int pitch, bool relu, bool valid, int m,
                                                int cbase, int h, const floatx16& acc,
                                                const half4 (&res)[4], bool has_res) {
  uint32_t q[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float v[4] = {acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]};
    if (has_res) {
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] += (float)res[i][j];
    }
    if (relu) {
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = fmaxf(v[j], 0.0f);
    }
    half4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (f16)v[j];
    const uint2 w = __builtin_bit_cast(uint2, o);
    q[i][0] = w.x;
    q[i][1] = w.y;
  }
#pragma unroll
  for (int pr = 0; pr < 2; ++pr)
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      const auto sw = __builtin_amdgcn_permlane32_swap(q[2 * pr][w], q[2 * pr + 1][w], false, false);
      q[2 * pr][w] = sw[0];
      q[2 * pr + 1][w] = sw[1];
    }
  if (valid) {
    f16* dst = out + (size_t)m * pitch + cbase + h * 8;
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      const u32x4 o = {q[2 * pr][0], q[2 * pr][1], q[2 * pr + 1][0], q[2 * pr + 1][1]};
      *reinterpret_cast<u32x4*>(dst + 16 * pr) = o;
    }
  }
}
__device__ __forceinline__ void store_octets(const ConvParams& p, bool valid, int m, int cbase,
                                             int h, const floatx16& acc, const half4 (&res)[4],
                                             bool has_res) {
  store_octets_to(p.out, p.out_pitch, p.relu != 0, valid, m, cbase, h, acc, res, has_res);
}
// The residual of a pixel's 32 channels, fetched the way store_octets stores them: lane half h
// loads channels cbase + 8h .. +7 and cbase + 16 + 8h .. +7 (two 16-byte loads, o[0] and o[1],
// from pixel_base + cbase + 8 * h and 16 halves further); the same lane exchange (it is its own
// inverse) turns them into the quads res[i] = channels cbase + 4h + 8i .. +3 that the
// accumulators are laid out in.  Every lane of the wavefront must call it.
__device__ __forceinline__ void res_octets_to_quads(const u32x4 (&o)[2], half4 (&res)[4]) {
  uint32_t q[4][2] = {{o[0][0], o[0][1]}, {o[0][2], o[0][3]}, {o[1][0], o[1][1]}, {o[1][2], o[1][3]}};
#pragma unroll
  for (int pr = 0; pr < 2; ++pr)
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      const auto sw = __builtin_amdgcn_permlane32_swap(q[2 * pr][w], q[2 * pr + 1][w], false, false);
      q[2 * pr][w] = sw[0];
      q[2 * pr + 1][w] = sw[1];
    }
#pragma unroll
  for (int i = 0; i < 4; ++i) res[i] = __builtin_bit_cast(half4, make_uint2(q[i][0], q[i][1]));
}

template <int KC, int DEPTH>
__global__ __launch_bounds__(256) void k_conv_mfma(ConvParams p) {
  constexpr int BM = 64, BN = 64;
  constexpr int PITCH = KC + 8;            // halves; +16 bytes keeps ds_read_b128 conflict-free
  constexpr int VPR = KC / 8;              // 16-byte vectors per tile row
  constexpr int NV = BM * VPR;             // vectors per tile (pixel tile and weight tile alike)
  constexpr int NP = (NV + 255) / 256;     // vectors per thread
  __shared__ __align__(16) f16 s_x[2][BM * PITCH];
  __shared__ __align__(16) f16 s_w[2][BN * PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // XCD-aware tile order.  Workgroups are dealt round-robin to the 8 XCDs (workgroup id % 8),
  // each with its own L2.  Tile t = (id % 8) * tiles_per_xcd + id / 8 gives every XCD a run of
  // consecutive tiles (pixel tile fastest, then channel tile, then K split): the workgroups
  // that share a weight slice, and neighbouring pixel tiles, meet in the same L2.
  const int tile = (int)(blockIdx.x & 7u) * p.tiles_per_xcd + (int)(blockIdx.x >> 3);
  if (tile >= p.tiles_m * p.tiles_n * p.nsplit) return;
  const int tile_m = tile % p.tiles_m;
  const int tile_n = (tile / p.tiles_m) % p.tiles_n;
  const int split = tile / (p.tiles_m * p.tiles_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int q_begin = split * p.chunks_per_split;
  const int q_end = min(p.nchunks, q_begin + p.chunks_per_split);

  // Per-thread loader state, fixed over the K loop: for every 16-byte vector this thread
  // fetches, the address of tap (0,0) / channel 0 of its pixel, the address of its weight
  // row, and one validity bit per tap (zero padding, ragged last tile).  Per chunk only a
  // wave-uniform offset is added, so the inner loop carries almost no address arithmetic.
  const f16* l_abase[NP];
  const f16* l_wbase[NP];
  uint32_t l_tapmask[NP];
  int l_lds[NP];
  bool l_act[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int v = tid + i * 256;
    l_act[i] = v < NV;
    const int row = (v / VPR) % BM;      // threads beyond the tile re-load a valid row, unused
    const int kv = v % VPR;
    const int m = m0 + row;
    const int img = m / p.img_m, ml = m - img * p.img_m;   // image of the batch, pixel in it
    const int oy = ml / p.wout, ox = ml - oy * p.wout;
    const int iy0 = oy * p.stride - p.pad, ix0 = ox * p.stride - p.pad;
    uint32_t mask = 0;
    for (int t = 0; t < p.ntaps; ++t) {
      const int ky = t / p.kw, kx = t - ky * p.kw;
      const int iy = iy0 + ky, ix = ix0 + kx;
      if (m < p.m && iy >= 0 && iy < p.hin && ix >= 0 && ix < p.win) mask |= 1u << t;
    }
    l_tapmask[i] = mask;
    l_abase[i] = p.in + (((long)img * p.hin + iy0) * p.win + ix0) * p.cin_pitch + kv * 8;
    l_wbase[i] = p.wt + (size_t)(n0 + row) * p.ktot + kv * 8;
    l_lds[i] = row * PITCH + kv * 8;
  }
  const f16* const a_safe = p.in;         // any valid address: out-of-range taps read it, unused

  // Loads are unconditional (out-of-range taps read a valid dummy address and are zeroed
  // when handed to LDS): with no branch around a load the compiler can count outstanding
  // loads exactly and waits only for the oldest stage.  Stage registers are indexed with
  // compile-time constants only (macro, fully unrolled) so that they stay in VGPRs.
  // Chunks are fetched strictly in order; (ld_q, ld_tap, ld_cc, ld_ky, ld_kx) is the next one
  // and stops advancing at the last chunk of this workgroup's range.
  u32x4 st_x[DEPTH][NP], st_w[DEPTH][NP];
  uint32_t st_inb[DEPTH];
  int ld_q = q_begin;
  int ld_tap = q_begin / p.chunks_per_tap;
  int ld_cc = q_begin - ld_tap * p.chunks_per_tap;
  int ld_ky = ld_tap / p.kw, ld_kx = ld_tap - ld_ky * p.kw;
#define HS_LOAD_CHUNK(D_)                                                                      \
  {                                                                                            \
    const long a_off_ = ((long)ld_ky * p.win + ld_kx) * p.cin_pitch + ld_cc * KC;              \
    const long w_off_ = (long)ld_q * KC;                                                       \
    uint32_t mask_ = 0;                                                                        \
    _Pragma("unroll") for (int i = 0; i < NP; ++i) {                                           \
      const bool inb_ = (l_tapmask[i] >> ld_tap) & 1u;                                         \
      mask_ |= (inb_ ? 1u : 0u) << i;                                                          \
      const f16* a_ = inb_ ? l_abase[i] + a_off_ : a_safe;                                     \
      st_x[D_][i] = *reinterpret_cast<const u32x4*>(a_);                                       \
      st_w[D_][i] = *reinterpret_cast<const u32x4*>(l_wbase[i] + w_off_);                      \
    }                                                                                          \
    st_inb[D_] = mask_;                                                                        \
    const bool adv_ = ld_q + 1 < q_end;                                                        \
    const bool wrap_c_ = ld_cc + 1 == p.chunks_per_tap;                                        \
    const bool wrap_x_ = wrap_c_ && (ld_kx + 1 == p.kw);                                       \
    ld_q += adv_ ? 1 : 0;                                                                      \
    ld_cc = !adv_ ? ld_cc : (wrap_c_ ? 0 : ld_cc + 1);                                         \
    ld_tap += (adv_ && wrap_c_) ? 1 : 0;                                                       \
    ld_ky += (adv_ && wrap_x_) ? 1 : 0;                                                        \
    ld_kx = !(adv_ && wrap_c_) ? ld_kx : (wrap_x_ ? 0 : ld_kx + 1);                            \
  }

  floatx16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.0f;

  const int wm = wave & 1, wn = wave >> 1;
  const int fx_off = (wm * 32 + (lane & 31)) * PITCH + (lane >> 5) * 8;
  const int fw_off = (wn * 32 + (lane & 31)) * PITCH + (lane >> 5) * 8;

  static_assert(DEPTH == 4 || DEPTH == 8, "the pipeline below is written out for 4 or 8 stages");
  // Prologue: fill all four stages.  Chunk indices are clamped instead of guarded so that
  // there is no branch around a load (a short K range re-loads its last chunk, unused).
  HS_LOAD_CHUNK(0)
  HS_LOAD_CHUNK(1)
  HS_LOAD_CHUNK(2)
  HS_LOAD_CHUNK(3)
  if constexpr (DEPTH > 4) {
    HS_LOAD_CHUNK(4)
    HS_LOAD_CHUNK(5)
    HS_LOAD_CHUNK(6)
    HS_LOAD_CHUNK(7)
  }

  // One pipeline step for stage D_ (a literal, so every register index is a constant):
  // hand chunk q to LDS, barrier, refill the stage with chunk q + DEPTH, MFMAs on chunk q.
  // REFILL_ is the refill condition: `true` in the steady-state loop (branch-free body, so
  // the wait before the LDS hand-over is for the oldest stage only), a test in the tail.
#define HS_STEP(D_, REFILL_)                                                                   \
  {                                                                                            \
    const int q = qb + (D_);                                                                   \
    (void)q;                                                                                   \
    _Pragma("unroll") for (int i = 0; i < NP; ++i) {                                           \
      if constexpr (NV % 256 != 0) { if (!l_act[i]) continue; }                                \
      const u32x4 zero = {0u, 0u, 0u, 0u};                                                     \
      *reinterpret_cast<u32x4*>(&s_x[buf][l_lds[i]]) =                                         \
          ((st_inb[D_] >> i) & 1u) ? st_x[D_][i] : zero;                                       \
      *reinterpret_cast<u32x4*>(&s_w[buf][l_lds[i]]) = st_w[D_][i];                            \
    }                                                                                          \
    __syncthreads();                                                                           \
    if (REFILL_) HS_LOAD_CHUNK(D_)                                                  \
    const f16* fx = &s_x[buf][fx_off];                                                         \
    const f16* fw = &s_w[buf][fw_off];                                                         \
    _Pragma("unroll") for (int ks = 0; ks < KC / 16; ++ks) {                                   \
      const half8 a = *reinterpret_cast<const half8*>(fw + ks * 16);                           \
      const half8 b = *reinterpret_cast<const half8*>(fx + ks * 16);                           \
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);                        \
    }                                                                                          \
    buf ^= 1;                                                                                  \
  }

  int buf = 0;
  int qb = q_begin;
  for (; qb + 2 * DEPTH <= q_end; qb += DEPTH) {   // steady state: every refill is in range
    HS_STEP(0, true)
    HS_STEP(1, true)
    HS_STEP(2, true)
    HS_STEP(3, true)
    if constexpr (DEPTH > 4) {
      HS_STEP(4, true)
      HS_STEP(5, true)
      HS_STEP(6, true)
      HS_STEP(7, true)
    }
  }
  for (; qb < q_end; qb += DEPTH) {                // tail: at most 2*DEPTH - 1 chunks
    if (qb + 0 < q_end) HS_STEP(0, q + DEPTH < q_end)
    if (qb + 1 < q_end) HS_STEP(1, q + DEPTH < q_end)
    if (qb + 2 < q_end) HS_STEP(2, q + DEPTH < q_end)
    if (qb + 3 < q_end) HS_STEP(3, q + DEPTH < q_end)
    if constexpr (DEPTH > 4) {
      if (qb + 4 < q_end) HS_STEP(4, q + DEPTH < q_end)
      if (qb + 5 < q_end) HS_STEP(5, q + DEPTH < q_end)
      if (qb + 6 < q_end) HS_STEP(6, q + DEPTH < q_end)
      if (qb + 7 < q_end) HS_STEP(7, q + DEPTH < q_end)
    }
  }
#undef HS_STEP

  // accumulator register 4*i + j holds channel n_base + 8*i + j of pixel m
  const int m = m0 + wm * 32 + (lane & 31);
  const int n_base = n0 + wn * 32 + (lane >> 5) * 4;
  if (!p.use_partial) {
    if (m >= p.m) return;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = n_base + 8 * i;
      if (n >= p.cout) continue;
      float v[4] = {acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]};
      store_quad(p, m, n, v);
    }
    return;
  }

  // ---- split-K: store fp32 partial sums; a separate kernel reduces them.  (Reducing inside
  // this kernel would need a device-wide release per workgroup, which on a multi-XCD part
  // means a full L2 write-back each time -- measured 3x slower than the extra launch.)
  if (m < p.m) {
    float* dst = p.partial + ((size_t)split * p.m + m) * p.cout_pad + n_base;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<float4*>(dst + 8 * i) =
          make_float4(acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]);
  }
}

#undef HS_LOAD_CHUNK

// =============================================================================================
// Stage 2, 3x3 stride-1 pad-1 layers (13 of the 21 convolutions, 85 % of the flops): the same
// implicit GEMM, but the workgroup's output tile is a SPATIAL block (8 rows x 8*MT columns),
// so that the nine taps read one shared (8+2) x (8*MT+2) input patch.  Per 64-channel chunk
// of Cin the patch goes to LDS once and serves all nine taps; only the weight tile (64 x 64
// halves per tap) is streamed per tap.  Global traffic per tap drops from 16 KB to
// 8 KB + patch/9 -- these layers are bound by bytes fetched per workgroup, not by MFMA rate.
// Pipeline: WS weight stages in registers (stage = tap % WS, a literal): while a tap is
// computed, the weights of the step WS taps ahead are being fetched -- with WS == 9 a whole
// chunk of weights is in flight, which suits grids of at most two workgroups per CU; the next
// chunk's patch is prefetched during the first taps of the current one and, with a single patch
// buffer (PB == 1), handed to LDS behind one extra barrier per chunk.  PB == 1 with WS == 3 is
// the lean form: 45 KB of LDS and under 170 registers, three workgroups per CU.  The nine steps
// of a chunk are written out, loads are unconditional and branch-free.
// Wavefront (wm, wn): pixel rows 4*wm .. 4*wm+3 (MT groups of 4 x 8 pixels), channels
// 32*wn .. +31.  chunks_per_split / nchunks count Cin chunks here (split-K over Cin).
// =============================================================================================
template <int MT, int PB, int WS, int STRIDE, bool PERSIST, int OCC>
__global__ __launch_bounds__(256, OCC) void k_conv3x3_halo(ConvParams p) {
  constexpr int KC = 64, TH = 8, TW = 8 * MT;
  constexpr int IPH = STRIDE * TH + 3 - STRIDE, IPW = STRIDE * TW + 3 - STRIDE;   // input patch
  constexpr int NPL = STRIDE * STRIDE;                 // parity planes the patch is stored as
  constexpr int PLH = STRIDE == 1 ? IPH : TH + 1, PLW = STRIDE == 1 ? IPW : TW + 1;
  constexpr int NPIX = IPH * IPW;
  constexpr int PITCH = KC + 8;
  constexpr int BN = 64;                     // output channels per workgroup
  constexpr int WL = BN / 32;                // weight vectors per thread and tap
  // Plane rows are padded so that consecutive rows start 128 bytes apart modulo 256: the 16
  // lanes of one ds_read_b128 pass (two rows of 8 pixels, 144-byte pixel pitch) then fall into
  // 16 different 16-byte bank groups.
  constexpr int RP = (PLW * PITCH * 2 + ((128 - (PLW * PITCH * 2) % 256 + 256) % 256)) / 2;
  static_assert((RP * 2) % 256 == 128, "plane row pitch must be 128 mod 256 bytes");
  constexpr int PV = NPIX * 8;               // 16-byte vectors in a patch
  constexpr int PL = (PV + 255) / 256;       // patch vectors per thread (4, 6 or 10)
  constexpr int PT = (PL + 8) / 9;           // of which fetched per tap
  static_assert(PT <= 2, "patch prefetch is spread over the nine taps");
  static_assert(WS == 9 || WS == 3, "weight stages: a divisor of nine");
  static_assert(STRIDE == 1 || (MT == 1 && PB == 1), "stride 2: 8 x 8 tile, one patch buffer");
  __shared__ __align__(16) f16 s_patch[PB][NPL * PLH * RP];
  __shared__ __align__(16) f16 s_w[2][BN * PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, h = lane >> 5;
  const int tile = (int)(blockIdx.x & 7u) * p.tiles_per_xcd + (int)(blockIdx.x >> 3);
  // A workgroup owns tiles_per_wg consecutive spatial tiles of one channel tile (and K split)
  // and walks them in one software pipeline: the next tile's patch is prefetched during the
  // last chunk of the current one, so the cold start is paid once per workgroup.
  const int groups_m = (p.tiles_m + p.tiles_per_wg - 1) / p.tiles_per_wg;
  if (tile >= groups_m * p.tiles_n * p.nsplit) return;
  // Tile order inside a K split: blocks of n_block channel tiles; inside a block the channel
  // tile varies fastest, then the spatial tile.  n_block == 1: the workgroups of one L2 share
  // a weight slice and every L2 that holds a channel tile fetches the input; n_block ==
  // tiles_n: they share input patches and every L2 fetches all the weights.  The host picks
  // the block size that brings the fewest bytes into the eight L2s.
  const int within = tile % (groups_m * p.tiles_n);
  const int blk = groups_m * p.n_block, in_blk = within % blk;
  const int tm_begin = (in_blk / p.n_block) * p.tiles_per_wg;
  const int tm_end = PERSIST ? min(p.tiles_m, tm_begin + p.tiles_per_wg) : tm_begin + 1;
  const int tile_n = (within / blk) * p.n_block + in_blk % p.n_block;
  const int split = tile / (groups_m * p.tiles_n);
  const int tiles_img = p.tiles_m / p.batch;            // spatial tiles per image
  const int n0 = tile_n * BN;
  const int cc_begin = split * p.chunks_per_split;
  const int cc_end = min(p.chunks_per_tap, cc_begin + p.chunks_per_split);
  const bool has_proj = STRIDE == 2 && p.wt2 != nullptr;
  // A layer with a single Cin chunk uses the same nine weight tiles for every tile a workgroup
  // walks: with all nine held in the register stages they are fetched once per workgroup
  // instead of once per tile (at 12 frames per launch the stage-1 layers otherwise pull four
  // times more weight bytes than activation bytes from L2).
  const bool keep_w = PERSIST && WS == 9 && p.chunks_per_tap == 1;

  // loop-invariant loader state
  const f16* l_wbase[WL];
  const f16* l_w2base[WL];
  int l_wlds[WL];
#pragma unroll
  for (int i = 0; i < WL; ++i) {
    const int v = tid + 256 * i, row = v >> 3, kv = v & 7;
    l_wbase[i] = p.wt + (size_t)(n0 + row) * p.ktot + kv * 8;
    l_w2base[i] = has_proj ? p.wt2 + (size_t)(n0 + row) * (p.chunks_per_tap * KC) + kv * 8 : p.wt;
    l_wlds[i] = row * PITCH + kv * 8;
  }
  // patch loader: the LDS slot of every vector is fixed, its source depends on the tile.
  // l_pyx packs the vector's pixel inside the patch; a source is kept as an offset in halves
  // from p.in (below 2^31 by construction of the plan), negative when the pixel is padding.
  int l_plds[PL], l_pyx[PL];
#pragma unroll
  for (int i = 0; i < PL; ++i) {
    const int v = tid + 256 * i;
    const int pix = min(v >> 3, NPIX - 1), kv = v & 7;
    const int py = pix / IPW, px = pix - py * IPW;
    l_pyx[i] = py | (px << 8);
    // stride 2: pixel (py, px) goes to parity plane (py & 1, px & 1) at (py / 2, px / 2), so
    // that the lanes of a tap read neighbouring plane pixels, as for stride 1.  -1: no such vector
    l_plds[i] = v >= PV ? -1
                : STRIDE == 1 ? py * RP + px * PITCH + kv * 8
                              : (((py & 1) * 2 + (px & 1)) * PLH + (py >> 1)) * RP +
                                    (px >> 1) * PITCH + kv * 8;
  }
  // source offsets of spatial tile TM_ (also its image and origin)
#define HS_TILE_SETUP(TM_, POFF_, IMG_, Y0_, X0_)                                              \
  {                                                                                            \
    IMG_ = (TM_) / tiles_img;                                                                  \
    const int ts_ = (TM_) - IMG_ * tiles_img;                                                  \
    const int ty_ = ts_ / p.tiles_x;                                                           \
    Y0_ = ty_ * TH;                                                                            \
    X0_ = (ts_ - ty_ * p.tiles_x) * TW;                                                        \
    _Pragma("unroll") for (int i = 0; i < PL; ++i) {                                           \
      const int iy_ = STRIDE * Y0_ + (l_pyx[i] & 0xff) - 1;                                    \
      const int ix_ = STRIDE * X0_ + (l_pyx[i] >> 8) - 1;                                      \
      const bool inb_ = l_plds[i] >= 0 && iy_ >= 0 && iy_ < p.hin && ix_ >= 0 && ix_ < p.win;  \
      POFF_[i] = inb_ ? ((IMG_ * p.hin + iy_) * p.win + ix_) * p.cin_pitch + (tid & 7) * 8 : -1; \
    }                                                                                          \
  }
  int l_poff[PL], l_poff_n[PL];
  int img, y0, x0, img_n, y0_n, x0_n;
  HS_TILE_SETUP(tm_begin, l_poff, img, y0, x0)

  const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  floatx16 acc[MT], acc2 = zero16;
#pragma unroll
  for (int g = 0; g < MT; ++g) acc[g] = zero16;

  const int wm = wave & 1, wn = wave >> 1;
  // fragment bases: weights row (32*wn + r); pixel (4*wm + r/8, r%8) of column group g
  const int fw_off = (wn * 32 + r) * PITCH + h * 8;
  const int fp_off = (4 * wm + (r >> 3)) * RP + (r & 7) * PITCH + h * 8;

  u32x4 st_w[WS][WL];
  u32x4 st_w2[WL];
  u32x4 st_p[PL];
#define HS_LOAD_W(S_, CC_, TAP_)                                                               \
  {                                                                                            \
    const long off_ = ((long)(TAP_) * p.chunks_per_tap + (CC_)) * KC;                          \
    _Pragma("unroll") for (int i = 0; i < WL; ++i)                                             \
      st_w[S_][i] = *reinterpret_cast<const u32x4*>(l_wbase[i] + off_);                        \
  }
#define HS_LOAD_W2(CC_)                                                                        \
  _Pragma("unroll") for (int i = 0; i < WL; ++i)                                               \
    st_w2[i] = *reinterpret_cast<const u32x4*>(l_w2base[i] + (long)(CC_) * KC);
#define HS_LOAD_P(I_, CC_, POFF_)                                                              \
  st_p[I_] = *reinterpret_cast<const u32x4*>(p.in + (POFF_[I_] >= 0 ? POFF_[I_] + (CC_) * KC : 0));
  // offset of tap (ky, kx) inside the patch, relative to the wavefront's first pixel
#define HS_TAP_OFF(KY_, KX_)                                                                   \
  (STRIDE == 1 ? (KY_) * RP + (KX_) * PITCH                                                    \
               : ((((KY_) & 1) * 2 + ((KX_) & 1)) * PLH + ((KY_) >> 1)) * RP + ((KX_) >> 1) * PITCH)

  // One tap of chunk cc of the current tile.  TAP_ and LAST_ are literals: every register index
  // and every refill decision is resolved at compile time.  Weight stage TAP_ % WS is handed to
  // LDS and refilled with the weights of the step WS taps ahead; CCN_, PBASE_N_, PINB_N_ name
  // the item after this chunk (next chunk of this tile, or first chunk of the next tile).
#define HS_TAP(TAP_, LAST_, CCN_, POFF_N_)                                                     \
  {                                                                                            \
    _Pragma("unroll") for (int i = 0; i < WL; ++i)                                             \
      *reinterpret_cast<u32x4*>(&s_w[buf][l_wlds[i]]) = st_w[(TAP_) % WS][i];                  \
    if ((TAP_) == 0) {                                                                         \
      if (PB == 1) __syncthreads(); /* every wave is done with the previous chunk's patch */   \
      const u32x4 zero_ = {0u, 0u, 0u, 0u};                                                    \
      _Pragma("unroll") for (int i = 0; i < PL; ++i)                                           \
        if (l_plds[i] >= 0)                                                                    \
          *reinterpret_cast<u32x4*>(&s_patch[pb][l_plds[i]]) = l_poff[i] >= 0 ? st_p[i] : zero_; \
    }                                                                                          \
    __syncthreads();                                                                           \
    if ((!(LAST_) || (TAP_) + WS < 9) && !keep_w)                                              \
      HS_LOAD_W((TAP_) % WS, ((TAP_) + WS >= 9 ? (CCN_) : cc), ((TAP_) + WS) % 9)              \
    if (!(LAST_)) {                                                                            \
      _Pragma("unroll") for (int i = PT * (TAP_); i < PT * (TAP_) + PT; ++i)                   \
        if (i < PL) { HS_LOAD_P(i < PL ? i : 0, CCN_, POFF_N_) }                               \
    }                                                                                          \
    const f16* fw_ = &s_w[buf][fw_off];                                                        \
    const f16* fp_ = &s_patch[pb][fp_off + HS_TAP_OFF((TAP_) / 3, (TAP_) % 3)];                \
    _Pragma("unroll") for (int ks = 0; ks < KC / 16; ++ks) {                                   \
      const half8 a_ = *reinterpret_cast<const half8*>(fw_ + ks * 16);                         \
      _Pragma("unroll") for (int g = 0; g < MT; ++g) {                                         \
        const half8 b_ = *reinterpret_cast<const half8*>(fp_ + g * 8 * PITCH + ks * 16);       \
        acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a_, b_, acc[g], 0, 0, 0);              \
      }                                                                                        \
    }                                                                                          \
    buf ^= 1;                                                                                  \
  }
  // Tenth step of a stride-2 chunk: the 1x1 stride-2 projection of the same input reads exactly
  // the centre tap's pixels, so it rides along with its own weights and accumulator.
#define HS_PROJ(LAST_, CCN_)                                                                   \
  if (has_proj) {                                                                              \
    _Pragma("unroll") for (int i = 0; i < WL; ++i)                                             \
      *reinterpret_cast<u32x4*>(&s_w[buf][l_wlds[i]]) = st_w2[i];                              \
    __syncthreads();                                                                           \
    if (!(LAST_)) { HS_LOAD_W2(CCN_) }                                                         \
    const f16* fw_ = &s_w[buf][fw_off];                                                        \
    const f16* fp_ = &s_patch[pb][fp_off + HS_TAP_OFF(1, 1)];                                  \
    _Pragma("unroll") for (int ks = 0; ks < KC / 16; ++ks) {                                   \
      const half8 a_ = *reinterpret_cast<const half8*>(fw_ + ks * 16);                         \
      const half8 b_ = *reinterpret_cast<const half8*>(fp_ + ks * 16);                         \
      acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a_, b_, acc2, 0, 0, 0);                    \
    }                                                                                          \
    buf ^= 1;                                                                                  \
  }
#define HS_CHUNK(LAST_, CCN_, PO_N_)                                                           \
  HS_TAP(0, LAST_, CCN_, PO_N_) HS_TAP(1, LAST_, CCN_, PO_N_) HS_TAP(2, LAST_, CCN_, PO_N_)    \
  HS_TAP(3, LAST_, CCN_, PO_N_) HS_TAP(4, LAST_, CCN_, PO_N_) HS_TAP(5, LAST_, CCN_, PO_N_)    \
  HS_TAP(6, LAST_, CCN_, PO_N_) HS_TAP(7, LAST_, CCN_, PO_N_) HS_TAP(8, LAST_, CCN_, PO_N_)    \
  if (STRIDE == 2) { HS_PROJ(LAST_, CCN_) }

  const int wm_rows = 4 * wm + (r >> 3);
  const int n_base = n0 + wn * 32 + h * 4;
  // The residual of a block's second convolution is fetched while the tile's last chunk is
  // still being computed, not between the last MFMA and the store (one full memory latency
  // at the end of every such launch otherwise).  Loads are unconditional, from clamped addresses.
  const bool res_here = p.res != nullptr && !p.use_partial;
  // fp16 output with whole 64-channel tiles: 16-byte stores after a lane exchange (store_octets);
  // not in the tile-walking stride-2 instantiation, which has no registers to spare for it
  const bool wide_out =
      !(STRIDE == 2 && PERSIST) && !p.use_partial && p.out_f32 == nullptr && (p.cout & 63) == 0;
  half4 res_pre[MT][4];
#define HS_RES_PREFETCH()                                                                      \
  if (res_here) {                                                                              \
    const int oy_ = min(y0 + wm_rows, p.hout - 1);                                             \
    _Pragma("unroll") for (int g = 0; g < MT; ++g) {                                           \
      const int ox_ = min(x0 + 8 * g + (r & 7), p.wout - 1);                                   \
      const f16* rp_ = p.res + (size_t)(img * p.img_m + oy_ * p.wout + ox_) * p.res_pitch;     \
      _Pragma("unroll") for (int i = 0; i < 4; ++i)                                            \
        res_pre[g][i] = *reinterpret_cast<const half4*>(rp_ + min(n_base + 8 * i, p.cout - 4)); \
    }                                                                                          \
  }
  // Stores the finished tile (image img, origin y0, x0) and clears the accumulators.
  // Accumulator quad i of group g: channels n_base + 8*i .. +3 of pixel (oy, ox_g).
#define HS_STORE_TILE()                                                                        \
  {                                                                                            \
    const int oy = y0 + wm_rows;                                                               \
    _Pragma("unroll") for (int g = 0; g < MT; ++g) {                                           \
      const int ox = x0 + 8 * g + (r & 7);                                                     \
      if (oy < p.hout && ox < p.wout) {                                                        \
        const int m = img * p.img_m + oy * p.wout + ox;                                        \
        if (p.use_partial) {                                                                   \
          float* dst = p.partial + ((size_t)split * p.m + m) * p.cout_pad + n_base;            \
          _Pragma("unroll") for (int i = 0; i < 4; ++i)                                        \
            *reinterpret_cast<float4*>(dst + 8 * i) = make_float4(                             \
                acc[g][4 * i], acc[g][4 * i + 1], acc[g][4 * i + 2], acc[g][4 * i + 3]);       \
        } else if (!wide_out) {                                                                \
          _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                      \
            const int n = n_base + 8 * i;                                                      \
            if (n < p.cout) {                                                                  \
              float v[4] = {acc[g][4 * i], acc[g][4 * i + 1], acc[g][4 * i + 2],               \
                            acc[g][4 * i + 3]};                                                \
              if (res_here) {                                                                  \
                _Pragma("unroll") for (int j = 0; j < 4; ++j) v[j] += (float)res_pre[g][i][j]; \
              }                                                                                \
              store_quad<false>(p, m, n, v);                                                   \
            }                                                                                  \
          }                                                                                    \
        }                                                                                      \
      }                                                                                        \
      if (wide_out)   /* every lane takes part in the exchange */                              \
        store_octets(p, oy < p.hout && ox < p.wout, img * p.img_m + oy * p.wout + ox,          \
                     n0 + wn * 32, h, acc[g], res_pre[g], res_here);                           \
      acc[g] = zero16;                                                                         \
    }                                                                                          \
    if (has_proj) { /* projection output: no residual, no ReLU */                              \
      const int ox = x0 + (r & 7);                                                             \
      if (oy < p.hout && ox < p.wout) {                                                        \
        const int m = img * p.img_m + oy * p.wout + ox;                                        \
        if (p.use_partial) {                                                                   \
          float* dst = p.partial2 + ((size_t)split * p.m + m) * p.cout_pad + n_base;           \
          _Pragma("unroll") for (int i = 0; i < 4; ++i)                                        \
            *reinterpret_cast<float4*>(dst + 8 * i) = make_float4(                             \
                acc2[4 * i], acc2[4 * i + 1], acc2[4 * i + 2], acc2[4 * i + 3]);               \
        } else {                                                                               \
          _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                      \
            const int n = n_base + 8 * i;                                                      \
            if (n < p.cout) {                                                                  \
              half4 o;                                                                         \
              _Pragma("unroll") for (int j = 0; j < 4; ++j) o[j] = (f16)acc2[4 * i + j];       \
              *reinterpret_cast<half4*>(p.out2 + (size_t)m * p.out2_pitch + n) = o;            \
            }                                                                                  \
          }                                                                                    \
        }                                                                                      \
      }                                                                                        \
      acc2 = zero16;                                                                           \
    }                                                                                          \
  }

  int buf = 0, pb = 0;
  int cc = cc_begin;
#pragma unroll
  for (int i = 0; i < PL; ++i) HS_LOAD_P(i, cc, l_poff)
  HS_LOAD_W(0, cc, 0) HS_LOAD_W(1, cc, 1) HS_LOAD_W(2, cc, 2)
  if (WS == 9) {
    HS_LOAD_W(3 % WS, cc, 3) HS_LOAD_W(4 % WS, cc, 4) HS_LOAD_W(5 % WS, cc, 5)
    HS_LOAD_W(6 % WS, cc, 6) HS_LOAD_W(7 % WS, cc, 7) HS_LOAD_W(8 % WS, cc, 8)
  }
  if (STRIDE == 2) { HS_LOAD_W2(cc) }
  // Items = (tile, chunk) pairs in order; `_n` state describes the item after the current one.
  const int n_items = (tm_end - tm_begin) * (cc_end - cc_begin);
  int tm = tm_begin;
#pragma unroll
  for (int i = 0; i < PL; ++i) l_poff_n[i] = l_poff[i];
  img_n = img; y0_n = y0; x0_n = x0;
  for (int item = 0; item + 1 < n_items; ++item) {
    const bool cross = PERSIST && cc + 1 == cc_end;    // the next item starts a new tile
    const int cc_nx = cross ? cc_begin : cc + 1;
    if (cross) {
      HS_TILE_SETUP(tm + 1, l_poff_n, img_n, y0_n, x0_n)
      HS_RES_PREFETCH()
    }
    HS_CHUNK(false, cc_nx, l_poff_n)
    if (PB == 2) pb ^= 1;
    if (cross) {
      HS_STORE_TILE()
#pragma unroll
      for (int i = 0; i < PL; ++i) l_poff[i] = l_poff_n[i];
      img = img_n; y0 = y0_n; x0 = x0_n;
      ++tm;
    }
    cc = cc_nx;
  }
  HS_RES_PREFETCH()
  HS_CHUNK(true, cc, l_poff)
  HS_STORE_TILE()
#undef HS_RES_PREFETCH
#undef HS_STORE_TILE
#undef HS_CHUNK
#undef HS_PROJ
#undef HS_TAP
#undef HS_TAP_OFF
#undef HS_LOAD_P
#undef HS_LOAD_W2
#undef HS_LOAD_W
#undef HS_TILE_SETUP
}

// =============================================================================================
// 3x3 stride-1 layers with 64 input channels (one Cin chunk) on grids several times the device:
// the nine weight tiles of a workgroup's channel tile never change while it walks its spatial
// tiles, so they are made resident once -- taps 0..2 in LDS, taps 3..8 as MFMA fragments in
// registers (all nine in LDS would leave one workgroup per CU, all nine in registers none of
// the registers).  A tile then costs one patch hand-over (two barriers) and 72 MFMAs per
// wavefront with no weight traffic and no barrier between the taps.  Same tile, wavefront
// layout and accumulation order (tap-major, four K-steps of 16 per tap) as
// k_conv3x3_halo<2, 1, 9, 1, true, *>: results are bit-identical.
// =============================================================================================
__global__ __launch_bounds__(256, 2) void k_conv3x3_c64_walk(ConvParams p) {
  constexpr int TH = 8, TW = 16, IPH = TH + 2, IPW = TW + 2, NPIX = IPH * IPW;
  constexpr int PITCH = 64 + 8;
  constexpr int RP = (IPW * PITCH * 2 + ((128 - (IPW * PITCH * 2) % 256 + 256) % 256)) / 2;
  static_assert((RP * 2) % 256 == 128, "plane row pitch must be 128 mod 256 bytes");
  constexpr int PV = NPIX * 8, PL = (PV + 255) / 256;
  constexpr int LT = 3;                       // taps whose weights stay in LDS (the rest: registers)
  constexpr int WT = 64 * PITCH;              // halves of one weight tile in LDS
  static_assert(IPH * RP >= 2 * WT, "the patch buffer stages two weight tiles in the prologue");
  __shared__ __align__(16) f16 s_patch[IPH * RP];
  __shared__ __align__(16) f16 s_wk[LT * WT];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, h = lane >> 5;
  const int tile = (int)(blockIdx.x & 7u) * p.tiles_per_xcd + (int)(blockIdx.x >> 3);
  const int groups_m = (p.tiles_m + p.tiles_per_wg - 1) / p.tiles_per_wg;
  if (tile >= groups_m * p.tiles_n) return;
  const int blk = groups_m * p.n_block, in_blk = tile % blk;       // tile order: see k_conv3x3_halo
  const int tm_begin = (in_blk / p.n_block) * p.tiles_per_wg;
  const int tm_end = min(p.tiles_m, tm_begin + p.tiles_per_wg);
  const int n0 = ((tile / blk) * p.n_block + in_blk % p.n_block) * 64;
  const int tiles_img = p.tiles_m / p.batch;
  const int wm = wave & 1, wn = wave >> 1;
  const int fw_off = (wn * 32 + r) * PITCH + h * 8;
  const int fp_off = (4 * wm + (r >> 3)) * RP + (r & 7) * PITCH + h * 8;

  // ---- patch loader: LDS slot and pixel of every vector are fixed, the source depends on the tile
  int l_plds[PL], l_pyx[PL];
#pragma unroll
  for (int i = 0; i < PL; ++i) {
    const int v = tid + 256 * i;
    const int pix = min(v >> 3, NPIX - 1), py = pix / IPW, px = pix - py * IPW;
    l_pyx[i] = py | (px << 8);
    l_plds[i] = v >= PV ? -1 : py * RP + px * PITCH + (v & 7) * 8;
  }
  u32x4 st_p[PL];
  uint32_t st_inb = 0;          // bit i: vector i of the fetched patch lies inside the image
  int f_img = 0, f_y0 = 0, f_x0 = 0;   // image and origin of the tile whose patch is in st_p
#define HS_FETCH_PATCH(TM_)                                                                    \
  {                                                                                            \
    f_img = (TM_) / tiles_img;                                                                 \
    const int ts_ = (TM_) - f_img * tiles_img, ty_ = ts_ / p.tiles_x;                          \
    f_y0 = ty_ * TH;                                                                           \
    f_x0 = (ts_ - ty_ * p.tiles_x) * TW;                                                       \
    st_inb = 0;                                                                                \
    _Pragma("unroll") for (int i = 0; i < PL; ++i) {                                           \
      const int iy_ = f_y0 + (l_pyx[i] & 0xff) - 1, ix_ = f_x0 + (l_pyx[i] >> 8) - 1;          \
      const bool in_ = l_plds[i] >= 0 && iy_ >= 0 && iy_ < p.hin && ix_ >= 0 && ix_ < p.win;   \
      st_inb |= (in_ ? 1u : 0u) << i;                                                          \
      const int off_ = in_ ? ((f_img * p.hin + iy_) * p.win + ix_) * p.cin_pitch + (tid & 7) * 8 : 0; \
      st_p[i] = *reinterpret_cast<const u32x4*>(p.in + off_);                                  \
    }                                                                                          \
  }
  HS_FETCH_PATCH(tm_begin)

  // ---- weights: taps 0..2 into their LDS tiles; taps 3..8, two at a time, through the (still
  // unused) patch buffer into fragment registers
  half8 a_keep[9 - LT][4];
  {
    const int row0 = tid >> 3, kv = tid & 7;        // this thread's vectors: rows row0, row0 + 32
    const f16* w0 = p.wt + (size_t)(n0 + row0) * p.ktot + kv * 8;
    const f16* w1 = w0 + (size_t)32 * p.ktot;
    const int l0 = row0 * PITCH + kv * 8, l1 = l0 + 32 * PITCH;
    u32x4 sw[9][2];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      sw[t][0] = *reinterpret_cast<const u32x4*>(w0 + t * 64);
      sw[t][1] = *reinterpret_cast<const u32x4*>(w1 + t * 64);
    }
#pragma unroll
    for (int t = 0; t < LT; ++t) {
      *reinterpret_cast<u32x4*>(&s_wk[t * WT + l0]) = sw[t][0];
      *reinterpret_cast<u32x4*>(&s_wk[t * WT + l1]) = sw[t][1];
    }
#pragma unroll
    for (int pair = 0; pair < (9 - LT) / 2; ++pair) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        *reinterpret_cast<u32x4*>(&s_patch[j * WT + l0]) = sw[LT + 2 * pair + j][0];
        *reinterpret_cast<u32x4*>(&s_patch[j * WT + l1]) = sw[LT + 2 * pair + j][1];
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
          a_keep[2 * pair + j][ks] =
              *reinterpret_cast<const half8*>(&s_patch[j * WT + fw_off + ks * 16]);
      __syncthreads();
    }
  }

  const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int n_base = n0 + wn * 32 + h * 4;
  for (int tm = tm_begin; tm < tm_end; ++tm) {
    const int img = f_img, y0 = f_y0, x0 = f_x0;
    if (tm != tm_begin) __syncthreads();      // every wavefront is done with the previous patch
#pragma unroll
    for (int i = 0; i < PL; ++i) {
      const u32x4 zero = {0u, 0u, 0u, 0u};
      if (l_plds[i] >= 0)
        *reinterpret_cast<u32x4*>(&s_patch[l_plds[i]]) = ((st_inb >> i) & 1u) ? st_p[i] : zero;
    }
    __syncthreads();
    if (tm + 1 < tm_end) HS_FETCH_PATCH(tm + 1)
    // residual of this tile: fetched now, used after the MFMAs (clamped addresses, unconditional)
    const int oy = y0 + 4 * wm + (r >> 3);
    u32x4 res_raw[2][2];      // two 16-byte pieces per pixel (res_octets_to_quads)
    if (p.res) {
      const int oy_c = min(oy, p.hout - 1);
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        const int ox_c = min(x0 + 8 * g + (r & 7), p.wout - 1);
        const f16* rp = p.res + (size_t)(img * p.img_m + oy_c * p.wout + ox_c) * p.res_pitch +
                        n0 + wn * 32 + h * 8;
        res_raw[g][0] = *reinterpret_cast<const u32x4*>(rp);
        res_raw[g][1] = *reinterpret_cast<const u32x4*>(rp + 16);
      }
    }

    floatx16 acc[2] = {zero16, zero16};
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const f16* fp = &s_patch[fp_off + (tap / 3) * RP + (tap % 3) * PITCH];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const half8 a = tap < LT ? *reinterpret_cast<const half8*>(&s_wk[tap * WT + fw_off + ks * 16])
                                 : a_keep[tap < LT ? 0 : tap - LT][ks];
#pragma unroll
        for (int g = 0; g < 2; ++g) {
          const half8 b = *reinterpret_cast<const half8*>(fp + g * 8 * PITCH + ks * 16);
          acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[g], 0, 0, 0);
        }
      }
    }

    // fp16 output with a multiple of 64 channels (the host selects this kernel only then)
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const int ox = x0 + 8 * g + (r & 7);
      half4 res_q[4] = {};
      if (p.res) res_octets_to_quads(res_raw[g], res_q);
      store_octets(p, oy < p.hout && ox < p.wout, img * p.img_m + oy * p.wout + ox, n0 + wn * 32, h,
                   acc[g], res_q, p.res != nullptr);
    }
  }
#undef HS_FETCH_PATCH
}

// =============================================================================================
// A whole 64-channel BasicBlock in one launch: out = ReLU(conv_b(ReLU(conv_a(x))) + x), both
// convolutions 3x3 stride 1 pad 1, 64 -> 64 channels (one workgroup owns every channel of its
// tile, so the intermediate tensor need not leave the CU).  For small grids (one frame, a few
// frames): there a layer is a kernel boundary, a cold start and nine dependent steps, and the
// block costs one of each of the first two instead of two.
//
// Output tile 8 x 16.  conv_b needs the intermediate on 10 x 18 pixels, conv_a therefore the
// input on 12 x 20.  Phase A: the 180 intermediate pixels in row-major order form six groups of
// 32 (the last 12 lanes idle); wavefront (wm, wn) computes groups wm, wm + 2, wm + 4 for
// channels 32*wn .. +31 and writes them -- ReLU, rounded to fp16 exactly as the unfused layer
// stores them, zero outside the image (conv_b's padding) -- into LDS over the input patch.
// Phase B is the tile loop body of k_conv3x3_c64_walk on that patch.  The 18 weight tiles
// stream through nine register stages and a double-buffered LDS tile, one barrier per tap;
// every output accumulates tap-major with four K-steps of 16 per tap, as in the unfused
// kernels: results are bit-identical to two k_conv3x3_halo launches.
// p.wt / p.wt2: packed weights of conv_a / conv_b; p.res = p.in (the shortcut).
// =============================================================================================
__global__ __launch_bounds__(256, 2) void k_block64_fused(ConvParams p) {
  constexpr int TH = 8, TW = 16, YH = TH + 2, YW = TW + 2, XH = TH + 4, XW = TW + 4;
  constexpr int PITCH = 64 + 8;
  constexpr int RPY = (YW * PITCH * 2 + ((128 - (YW * PITCH * 2) % 256 + 256) % 256)) / 2;
  constexpr int RPX = (XW * PITCH * 2 + ((128 - (XW * PITCH * 2) % 256 + 256) % 256)) / 2;
  static_assert((RPY * 2) % 256 == 128 && (RPX * 2) % 256 == 128, "row pitch must be 128 mod 256 bytes");
  static_assert(XH * RPX >= YH * RPY, "the intermediate patch is written over the input patch");
  constexpr int NPY = YH * YW;                         // 180 intermediate pixels
  constexpr int XV = XH * XW * 8, XL = (XV + 255) / 256;   // input patch vectors, per thread
  constexpr int WT = 64 * PITCH;
  __shared__ __align__(16) f16 s_xy[XH * RPX];
  __shared__ __align__(16) f16 s_w[2 * WT];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, h = lane >> 5;
  const int tm = (int)(blockIdx.x & 7u) * p.tiles_per_xcd + (int)(blockIdx.x >> 3);
  if (tm >= p.tiles_m) return;
  const int tiles_img = p.tiles_m / p.batch;
  const int img = tm / tiles_img, ts = tm - img * tiles_img, ty = ts / p.tiles_x;
  const int y0 = ty * TH, x0 = (ts - ty * p.tiles_x) * TW;
  const int wm = wave & 1, wn = wave >> 1;

  // ---- input patch: pixel (y0 - 2 + py, x0 - 2 + px), zeros outside the image
  u32x4 st_x[XL];
  uint32_t x_inb = 0;
#pragma unroll
  for (int i = 0; i < XL; ++i) {
    const int v = tid + 256 * i;
    const int pix = min(v >> 3, XH * XW - 1), py = pix / XW, px = pix - py * XW;
    const int iy = y0 - 2 + py, ix = x0 - 2 + px;
    const bool in = v < XV && iy >= 0 && iy < p.hin && ix >= 0 && ix < p.win;
    x_inb |= (in ? 1u : 0u) << i;
    const int off = in ? ((img * p.hin + iy) * p.win + ix) * p.cin_pitch + (tid & 7) * 8 : 0;
    st_x[i] = *reinterpret_cast<const u32x4*>(p.in + off);
  }
  // ---- weights: stage t holds tap t of conv_a, later tap t of conv_b
  const int w_row = tid >> 3, w_kv = tid & 7;
  const f16* wa0 = p.wt + (size_t)w_row * p.ktot + w_kv * 8;
  const f16* wa1 = wa0 + (size_t)32 * p.ktot;
  const f16* wb0 = p.wt2 + (size_t)w_row * p.ktot + w_kv * 8;
  const f16* wb1 = wb0 + (size_t)32 * p.ktot;
  const int wl0 = w_row * PITCH + w_kv * 8, wl1 = wl0 + 32 * PITCH;
  u32x4 st_w[9][2];
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    st_w[t][0] = *reinterpret_cast<const u32x4*>(wa0 + t * 64);
    st_w[t][1] = *reinterpret_cast<const u32x4*>(wa1 + t * 64);
  }
#pragma unroll
  for (int i = 0; i < XL; ++i) {
    const int v = tid + 256 * i;
    if (v < XV) {
      const int pix = v >> 3, py = pix / XW, px = pix - py * XW;
      const u32x4 zero = {0u, 0u, 0u, 0u};
      *reinterpret_cast<u32x4*>(&s_xy[py * RPX + px * PITCH + (v & 7) * 8]) =
          ((x_inb >> i) & 1u) ? st_x[i] : zero;
    }
  }

  const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int fw_off = (wn * 32 + r) * PITCH + h * 8;

  // ---- phase A: intermediate pixel q = 32*(wm + 2k) + r of the 10 x 18 patch, k = 0..2
  int a_py[3], a_px[3], a_off[3];
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    const int q = min(32 * (wm + 2 * k) + r, NPY - 1);
    a_py[k] = q / YW;
    a_px[k] = q - a_py[k] * YW;
    a_off[k] = a_py[k] * RPX + a_px[k] * PITCH + h * 8;
  }
  floatx16 acc_a[3] = {zero16, zero16, zero16};
#pragma unroll
  for (int tap = 0; tap < 9; ++tap) {
    f16* sw = &s_w[(tap & 1) * WT];
    *reinterpret_cast<u32x4*>(&sw[wl0]) = st_w[tap][0];
    *reinterpret_cast<u32x4*>(&sw[wl1]) = st_w[tap][1];
    __syncthreads();
    st_w[tap][0] = *reinterpret_cast<const u32x4*>(wb0 + tap * 64);
    st_w[tap][1] = *reinterpret_cast<const u32x4*>(wb1 + tap * 64);
    const int toff = (tap / 3) * RPX + (tap % 3) * PITCH;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const half8 a = *reinterpret_cast<const half8*>(&sw[fw_off + ks * 16]);
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        const half8 b = *reinterpret_cast<const half8*>(&s_xy[a_off[k] + toff + ks * 16]);
        acc_a[k] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc_a[k], 0, 0, 0);
      }
    }
  }
  __syncthreads();          // every wavefront is done with the input patch
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    const int q = 32 * (wm + 2 * k) + r;
    const int iy = y0 - 1 + a_py[k], ix = x0 - 1 + a_px[k];
    const bool inside = iy >= 0 && iy < p.hin && ix >= 0 && ix < p.win;
    if (q < NPY) {
      f16* dst = &s_xy[a_py[k] * RPY + a_px[k] * PITCH + wn * 32 + h * 4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        half4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = inside ? (f16)fmaxf(acc_a[k][4 * i + j], 0.0f) : (f16)0.0f;
        *reinterpret_cast<half4*>(dst + 8 * i) = o;
      }
    }
  }

  // ---- residual of this tile (the block's input), fetched now, used after phase B
  const int oy = y0 + 4 * wm + (r >> 3);
  const int n_base = wn * 32 + h * 4;
  half4 res_pre[2][4];
  {
    const int oy_c = min(oy, p.hout - 1);
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const int ox_c = min(x0 + 8 * g + (r & 7), p.wout - 1);
      const f16* rp = p.res + (size_t)(img * p.img_m + oy_c * p.wout + ox_c) * p.res_pitch;
#pragma unroll
      for (int i = 0; i < 4; ++i) res_pre[g][i] = *reinterpret_cast<const half4*>(rp + n_base + 8 * i);
    }
  }

  // ---- phase B: conv_b on the intermediate patch (the first barrier below also publishes it)
  const int fp_off = (4 * wm + (r >> 3)) * RPY + (r & 7) * PITCH + h * 8;
  floatx16 acc_b[2] = {zero16, zero16};
#pragma unroll
  for (int tap = 0; tap < 9; ++tap) {
    f16* sw = &s_w[((tap + 1) & 1) * WT];       // continues the alternation of phase A (taps 9..17)
    *reinterpret_cast<u32x4*>(&sw[wl0]) = st_w[tap][0];
    *reinterpret_cast<u32x4*>(&sw[wl1]) = st_w[tap][1];
    __syncthreads();
    const f16* fp = &s_xy[fp_off + (tap / 3) * RPY + (tap % 3) * PITCH];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const half8 a = *reinterpret_cast<const half8*>(&sw[fw_off + ks * 16]);
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        const half8 b = *reinterpret_cast<const half8*>(fp + g * 8 * PITCH + ks * 16);
        acc_b[g] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc_b[g], 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    const int ox = x0 + 8 * g + (r & 7);
    store_octets(p, oy < p.hout && ox < p.wout, img * p.img_m + oy * p.wout + ox, wn * 32, h,
                 acc_b[g], res_pre[g], true);
  }
}

// =============================================================================================
// 3x3 stride-1 pad-1 layers with several Cin chunks on grids of at least 1.5 workgroups per CU
// (stages 2-4 and the ConvLSTM gates from a few frames per launch on).  Same 8 x 16 spatial
// tile, wavefront layout and accumulation order as k_conv3x3_halo<2, ...> -- bit-identical
// results -- but the weights never touch LDS: they are packed on the host in MFMA fragment
// order (one 1 KB block of 64 lanes x 16 bytes per 32 channels, tap and K-step of 16) and every
// wavefront loads its "A" fragments straight into registers, three taps ahead.  On those grids
// the layers are paced by LDS throughput (a tap step of the LDS-staged kernel moves 48 KB of
// fragment reads and 10 KB of writes per workgroup; writes run at under half the rate of
// reads): without the weight tile the LDS carries the pixel fragments only (32 KB of reads per
// tap step), the per-tap barrier disappears (one barrier per Cin chunk, for the patch), and
// the weight bytes come through the vector memory path, which has room (16 KB per tap step
// and workgroup; the two wavefronts that share a channel half fetch the same lines).
// The input patch is double buffered: chunk c+1 streams into the other buffer during the
// taps of chunk c, at most four vectors per thread in flight.
// p.wt_frag: [cout_pad / 32][Cin chunk][tap][K-step][lane][8 halves]; a workgroup's K range is
// one contiguous run per channel half, walked by a pointer that advances 4 KB per tap.
// =============================================================================================
__global__ __launch_bounds__(256, 3) void k_conv3x3_dira(ConvParams p) {
  constexpr int KC = 64, TH = 8, TW = 16, IPH = TH + 2, IPW = TW + 2, NPIX = IPH * IPW;
  constexpr int PITCH = KC + 8;
  constexpr int RP = (IPW * PITCH * 2 + ((128 - (IPW * PITCH * 2) % 256 + 256) % 256)) / 2;
  static_assert((RP * 2) % 256 == 128, "plane row pitch must be 128 mod 256 bytes");
  constexpr int PV = NPIX * 8;               // 16-byte vectors in a patch
  constexpr int PL = (PV + 255) / 256;       // patch vectors per thread
  static_assert(PL == 6, "the patch pipeline below is written out for six vectors per thread");
  __shared__ __align__(16) f16 s_patch[2][IPH * RP];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, h = lane >> 5;
  const int tile = (int)(blockIdx.x & 7u) * p.tiles_per_xcd + (int)(blockIdx.x >> 3);
  if (tile >= p.tiles_m * p.tiles_n * p.nsplit) return;
  const int within = tile % (p.tiles_m * p.tiles_n);              // tile order: see k_conv3x3_halo
  const int blk = p.tiles_m * p.n_block, in_blk = within % blk;
  const int tm = in_blk / p.n_block;
  const int tile_n = (within / blk) * p.n_block + in_blk % p.n_block;
  const int split = tile / (p.tiles_m * p.tiles_n);
  const int tiles_img = p.tiles_m / p.batch;
  const int n0 = tile_n * 64;
  const int cc_begin = split * p.chunks_per_split;
  const int cc_end = min(p.chunks_per_tap, cc_begin + p.chunks_per_split);
  const int img = tm / tiles_img, ts = tm - img * tiles_img, ty = ts / p.tiles_x;
  const int y0 = ty * TH, x0 = (ts - ty * p.tiles_x) * TW;
  const int wm = wave & 1, wn = wave >> 1;

  // ---- patch loader: LDS slot and source offset (in halves from p.in, -1: padding) per vector
  int l_plds[PL], l_poff[PL];
#pragma unroll
  for (int i = 0; i < PL; ++i) {
    const int v = tid + 256 * i;
    const int pix = min(v >> 3, NPIX - 1), py = pix / IPW, px = pix - py * IPW;
    l_plds[i] = v >= PV ? -1 : py * RP + px * PITCH + (v & 7) * 8;
    const int iy = y0 + py - 1, ix = x0 + px - 1;
    const bool inb = v < PV && iy >= 0 && iy < p.hin && ix >= 0 && ix < p.win;
    l_poff[i] = inb ? ((img * p.hin + iy) * p.win + ix) * p.cin_pitch + (tid & 7) * 8 : -1;
  }
#define HS_LOAD_P(I_, CC_) \
  st_p[(I_) & 3] = *reinterpret_cast<const u32x4*>(p.in + (l_poff[I_] >= 0 ? l_poff[I_] + (CC_) * KC : 0));
#define HS_HAND_P(I_, PB_)                                                                     \
  if (l_plds[I_] >= 0) {                                                                       \
    const u32x4 zero_ = {0u, 0u, 0u, 0u};                                                      \
    *reinterpret_cast<u32x4*>(&s_patch[PB_][l_plds[I_]]) = l_poff[I_] >= 0 ? st_p[(I_) & 3] : zero_; \
  }
  u32x4 st_p[4];

  // ---- weight fragments: this wavefront's 32 channels, one 1 KB block per (chunk, tap, K-step)
  const u32x4* wf = reinterpret_cast<const u32x4*>(p.wt_frag) +
                    ((size_t)(n0 / 32 + wn) * p.chunks_per_tap + cc_begin) * (9 * 4 * 64) + lane;
  const u32x4* const wf_last = wf + (size_t)((cc_end - cc_begin) * 9 - 1) * (4 * 64);
  u32x4 fa[3][4];
#define HS_LOAD_A(S_)                                                                          \
  {                                                                                            \
    _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) fa[S_][ks] = wf[ks * 64];                 \
    wf = wf + 4 * 64 <= wf_last ? wf + 4 * 64 : wf_last;   /* the last steps re-read the last tap */ \
  }

  const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  floatx16 acc[2] = {zero16, zero16};
  const int fp_off = (4 * wm + (r >> 3)) * RP + (r & 7) * PITCH + h * 8;

  // A chunk is 36 K-steps of 16 (tap-major, four per tap); Q_ and LAST_ are literals.  Weight
  // stage (Q_ / 4) % 3 holds the tap's fragments and is refilled, behind their last use, with
  // those of the step three taps ahead.  Pixel fragments are read from LDS BD K-steps before
  // the MFMAs that use them (a ring of BD + 1 register sets), so that an LDS round trip hides
  // behind 2 * BD MFMAs of this wavefront; only the first BD steps of a chunk, behind its
  // barrier, wait for theirs.  Vector i of the next chunk's patch is fetched at tap i and
  // handed to the other buffer at tap i + 3.
  constexpr int BD = 3;
  half8 bf[BD + 1][2];
#define HS_READ_B(Q_)                                                                          \
  {                                                                                            \
    const f16* fp_ = &s_patch[pb][fp_off + ((Q_) / 12) * RP + (((Q_) / 4) % 3) * PITCH + ((Q_) % 4) * 16]; \
    _Pragma("unroll") for (int g = 0; g < 2; ++g)                                              \
      bf[(Q_) % (BD + 1)][g] = *reinterpret_cast<const half8*>(fp_ + g * 8 * PITCH);           \
  }
#define HS_KSTEP(Q_, LAST_)                                                                    \
  {                                                                                            \
    if ((Q_) + BD < 36) HS_READ_B((Q_) + BD)                                                   \
    if ((Q_) % 4 == 0) {                                                                       \
      if (!(LAST_) && (Q_) / 4 >= 3) HS_HAND_P((Q_) / 4 - 3, pb ^ 1)                           \
      if (!(LAST_) && (Q_) / 4 < PL) HS_LOAD_P((Q_) / 4, cc + 1)                               \
    }                                                                                          \
    const half8 a_ = __builtin_bit_cast(half8, fa[((Q_) / 4) % 3][(Q_) % 4]);                  \
    _Pragma("unroll") for (int g = 0; g < 2; ++g)                                              \
      acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a_, bf[(Q_) % (BD + 1)][g], acc[g], 0, 0, 0); \
    if ((Q_) % 4 == 3) HS_LOAD_A(((Q_) / 4) % 3)                                               \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  }
#define HS_TAP(T_, LAST_)                                                                      \
  HS_KSTEP(4 * (T_), LAST_) HS_KSTEP(4 * (T_) + 1, LAST_) HS_KSTEP(4 * (T_) + 2, LAST_)        \
  HS_KSTEP(4 * (T_) + 3, LAST_)
#define HS_CHUNK(LAST_)                                                                        \
  HS_READ_B(0) HS_READ_B(1) HS_READ_B(2)                                                       \
  HS_TAP(0, LAST_) HS_TAP(1, LAST_) HS_TAP(2, LAST_) HS_TAP(3, LAST_) HS_TAP(4, LAST_)         \
  HS_TAP(5, LAST_) HS_TAP(6, LAST_) HS_TAP(7, LAST_) HS_TAP(8, LAST_)
  static_assert(BD == 3, "HS_CHUNK primes three K-steps");

  // ---- prologue: first patch into buffer 0, first three taps of weights into the stages
  int cc = cc_begin, pb = 0;
  {
    u32x4 first[PL];
#pragma unroll
    for (int i = 0; i < PL; ++i)
      first[i] = *reinterpret_cast<const u32x4*>(p.in + (l_poff[i] >= 0 ? l_poff[i] + cc * KC : 0));
    HS_LOAD_A(0) HS_LOAD_A(1) HS_LOAD_A(2)
#pragma unroll
    for (int i = 0; i < PL; ++i)
      if (l_plds[i] >= 0) {
        const u32x4 zero = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4*>(&s_patch[0][l_plds[i]]) = l_poff[i] >= 0 ? first[i] : zero;
      }
  }
  __syncthreads();

  const int oy = y0 + 4 * wm + (r >> 3);
  const int n_base = n0 + wn * 32 + h * 4;
  for (; cc + 1 < cc_end; ++cc) {
    HS_CHUNK(false)
    __syncthreads();      // the next patch is complete, and every wavefront is done with this one
    pb ^= 1;
  }
  // residual of the block's second convolution: fetched while the last chunk is computed
  // (with whole 64-channel tiles of fp16 output as two 16-byte pieces per pixel, see
  // res_octets_to_quads; otherwise as the four quads the accumulators are laid out in)
  const bool res_here = p.res != nullptr && !p.use_partial;
  const bool wide_out = !p.use_partial && p.out_f32 == nullptr && (p.cout & 63) == 0;
  half4 res_pre[2][4];
  u32x4 res_raw[2][2];
  if (res_here) {
    const int oy_c = min(oy, p.hout - 1);
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const int ox_c = min(x0 + 8 * g + (r & 7), p.wout - 1);
      const f16* rp = p.res + (size_t)(img * p.img_m + oy_c * p.wout + ox_c) * p.res_pitch;
      if (wide_out) {
        res_raw[g][0] = *reinterpret_cast<const u32x4*>(rp + n0 + wn * 32 + h * 8);
        res_raw[g][1] = *reinterpret_cast<const u32x4*>(rp + n0 + wn * 32 + h * 8 + 16);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          res_pre[g][i] = *reinterpret_cast<const half4*>(rp + min(n_base + 8 * i, p.cout - 4));
      }
    }
  }
  HS_CHUNK(true)

  // ---- epilogue: accumulator quad i of group g = channels n_base + 8*i .. +3 of pixel (oy, ox_g)
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    const int ox = x0 + 8 * g + (r & 7);
    const bool valid = oy < p.hout && ox < p.wout;
    const int m = img * p.img_m + oy * p.wout + ox;
    if (wide_out) {                       // every lane takes part in the exchanges
      if (res_here) res_octets_to_quads(res_raw[g], res_pre[g]);
      store_octets(p, valid, m, n0 + wn * 32, h, acc[g], res_pre[g], res_here);
    } else if (valid) {
      if (p.use_partial) {
        float* dst = p.partial + ((size_t)split * p.m + m) * p.cout_pad + n_base;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          *reinterpret_cast<float4*>(dst + 8 * i) =
              make_float4(acc[g][4 * i], acc[g][4 * i + 1], acc[g][4 * i + 2], acc[g][4 * i + 3]);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int n = n_base + 8 * i;
          if (n < p.cout) {
            float v[4] = {acc[g][4 * i], acc[g][4 * i + 1], acc[g][4 * i + 2], acc[g][4 * i + 3]};
            if (res_here) {
#pragma unroll
              for (int j = 0; j < 4; ++j) v[j] += (float)res_pre[g][i][j];
            }
            store_quad<false>(p, m, n, v);
          }
        }
      }
    }
  }
#undef HS_CHUNK
#undef HS_TAP
#undef HS_KSTEP
#undef HS_READ_B
#undef HS_LOAD_A
#undef HS_HAND_P
#undef HS_LOAD_P
}

// =============================================================================================
// 3x3 stride-2 pad-1 layers (with the block's 1x1 stride-2 projection riding along) on grids of
// at least 1.5 workgroups per CU: the stride-2 counterpart of k_conv3x3_dira.  Output tile 8 x 8
// pixels x 128 channels; wavefront w = all 64 pixels (two groups of four rows), channels
// 32*w .. +31: a weight fragment is fetched by one wavefront only and serves two MFMAs, and
// the patch -- the heavy operand of a stride-2 tile -- serves 128 channels.
// A stride-2 tile needs four input pixels per output pixel (17 x 17 of them), and with the
// weight tile in LDS and a barrier per tap a wavefront got four MFMAs per barrier: those layers
// ran the matrix pipe at 16-23 %.  Here
//   - the weights come as MFMA fragments straight from memory (p.wt_frag, and p.wt2_frag for the
//     projection), three taps ahead: no weight tile, no per-tap barrier;
//   - the patch is cut into half chunks of 32 input channels (one "item" = one half chunk of
//     one tile: nine taps + the projection, two K-steps of 16 each), stored as four parity
//     planes of 9 x 9 pixels (pixel (py, px) in plane (py & 1, px & 1) at (py / 2, px / 2), so that
//     the lanes of a tap read neighbouring plane pixels) with 64 bytes per pixel and no padding:
//     the four 16-byte vectors of a pixel are permuted by its plane row and column
//     (v ^ ((col >> 2) & 1 | (row & 1) << 1)), which makes every fragment read conflict free.
//     Two buffers of 20 KB: the next item's patch streams in during the taps of the current
//     one (four vectors per thread in flight), one barrier per item, two workgroups per CU
//     (four accumulators per wavefront with the projection's);
//   - a workgroup walks tiles_per_wg consecutive spatial tiles in one pipeline (the next tile's
//     first patch and weights are fetched during the last taps of the current tile), so the
//     short K loops of the 64-channel layer do not pay a cold start per tile.
// Per output the K order is chunk, half chunk, tap, K-step: within a chunk the two halves are
// summed one after the other, not interleaved tap by tap as in k_conv3x3_halo<1, 1, 3, 2, ...>;
// results agree with that kernel to fp32 rounding, not bit for bit.
// =============================================================================================
__global__ __launch_bounds__(256, 2) void k_conv3x3s2_dira(ConvParams p) {
  constexpr int TH = 8, TW = 8, IPW = 2 * TW + 1, NPIX = IPW * IPW;   // 17 x 17 input pixels
  constexpr int PLW = TW + 1, PLANE = PLW * PLW;                      // 9 x 9 pixels per parity plane
  constexpr int PV = NPIX * 4, PL = (PV + 255) / 256;                 // 16-byte vectors, per thread
  static_assert(PL == 5, "the patch pipeline below is written out for five vectors per thread");
  __shared__ __align__(16) f16 s_patch[2][4 * PLANE * 32];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, h = lane >> 5;
  const int tile = (int)(blockIdx.x & 7u) * p.tiles_per_xcd + (int)(blockIdx.x >> 3);
  const int groups_m = (p.tiles_m + p.tiles_per_wg - 1) / p.tiles_per_wg;
  if (tile >= groups_m * p.tiles_n * p.nsplit) return;
  const int within = tile % (groups_m * p.tiles_n);               // tile order: see k_conv3x3_halo
  const int blk = groups_m * p.n_block, in_blk = within % blk;
  const int tm_begin = (in_blk / p.n_block) * p.tiles_per_wg;
  const int tm_end = min(p.tiles_m, tm_begin + p.tiles_per_wg);
  const int tile_n = (within / blk) * p.n_block + in_blk % p.n_block;
  const int split = tile / (groups_m * p.tiles_n);
  const int tiles_img = p.tiles_m / p.batch;
  const int n0 = tile_n * 128;
  const int cc_begin = split * p.chunks_per_split;
  const int cc_end = min(p.chunks_per_tap, cc_begin + p.chunks_per_split);
  const int n_halves = 2 * (cc_end - cc_begin);                   // items per tile
  const int n_items = (tm_end - tm_begin) * n_halves;
  const bool has_proj = p.wt2_frag != nullptr;

  // ---- patch loader: the LDS slot of every vector is fixed, its source depends on the tile
  int l_plds[PL], l_pyx[PL], l_poff[PL];
#pragma unroll
  for (int i = 0; i < PL; ++i) {
    const int vec = tid + 256 * i, pix = min(vec >> 2, NPIX - 1), v = vec & 3;
    const int py = pix / IPW, px = pix - py * IPW, prow = py >> 1, pcol = px >> 1;
    const int sw = ((pcol >> 2) & 1) | ((prow & 1) << 1);
    l_pyx[i] = py | (px << 8);
    l_plds[i] = vec >= PV ? -1
                          : ((((py & 1) * 2 + (px & 1)) * PLANE + prow * PLW + pcol) * 4 + (v ^ sw)) * 8;
  }
  // source offsets (halves from p.in, channel 8 * (tid & 3) of the pixel; -1: padding) of tile TM_
#define HS_TILE_SETUP(TM_, IMG_, Y0_, X0_)                                                     \
  {                                                                                            \
    IMG_ = (TM_) / tiles_img;                                                                  \
    const int ts_ = (TM_) - IMG_ * tiles_img, ty_ = ts_ / p.tiles_x;                           \
    Y0_ = ty_ * TH;                                                                            \
    X0_ = (ts_ - ty_ * p.tiles_x) * TW;                                                        \
    _Pragma("unroll") for (int i = 0; i < PL; ++i) {                                           \
      const int iy_ = 2 * Y0_ + (l_pyx[i] & 0xff) - 1, ix_ = 2 * X0_ + (l_pyx[i] >> 8) - 1;    \
      const bool inb_ = l_plds[i] >= 0 && iy_ >= 0 && iy_ < p.hin && ix_ >= 0 && ix_ < p.win;  \
      l_poff[i] = inb_ ? ((IMG_ * p.hin + iy_) * p.win + ix_) * p.cin_pitch + (tid & 3) * 8 : -1; \
    }                                                                                          \
  }
  u32x4 st_p[4];
#define HS_LOAD_P(I_) \
  st_p[(I_) & 3] = *reinterpret_cast<const u32x4*>(p.in + (l_poff[I_] >= 0 ? l_poff[I_] + ch_n : 0));
#define HS_HAND_P(I_, PB_)                                                                     \
  if (l_plds[I_] >= 0) {                                                                       \
    const u32x4 zero_ = {0u, 0u, 0u, 0u};                                                      \
    *reinterpret_cast<u32x4*>(&s_patch[PB_][l_plds[I_]]) = l_poff[I_] >= 0 ? st_p[(I_) & 3] : zero_; \
  }

  // ---- pixel fragments: lane (r, h) reads output pixels (4*g + r/8, r%8), g = 0, 1; tap (ky, kx)
  // reads plane (ky & 1, kx & 1) at (+ky/2, +kx/2); K-step j of the item is vector 2*j + h of the
  // pixel.  Group 1 lies four plane rows below group 0 (same row parity, same permutation).
  constexpr int GOFF = 4 * PLW * 32;
  const int oy_l = r >> 3, ox_l = r & 7;
  int fb[2][2][2];    // [ky / 2][kx / 2][j]: halves offset inside a plane
#pragma unroll
  for (int dy = 0; dy < 2; ++dy)
#pragma unroll
    for (int dx = 0; dx < 2; ++dx) {
      const int prow = oy_l + dy, pcol = ox_l + dx;
      const int sw = ((pcol >> 2) & 1) | ((prow & 1) << 1);
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[dy][dx][j] = ((prow * PLW + pcol) * 4 + ((2 * j + h) ^ sw)) * 8;
    }

  // ---- weight fragments of this wavefront's 32 channels: blocks of 64 lanes x 16 bytes,
  // [chunk][tap][K-step of 16] for the 3x3 taps, [chunk][K-step] for the projection
  const u32x4* const wf0 = reinterpret_cast<const u32x4*>(p.wt_frag) +
                           (size_t)(n0 / 32 + wave) * p.chunks_per_tap * (9 * 4 * 64) + lane;
  const u32x4* const wp0 = has_proj ? reinterpret_cast<const u32x4*>(p.wt2_frag) +
                                          (size_t)(n0 / 32 + wave) * p.chunks_per_tap * (4 * 64) + lane
                                    : wf0;
  // half chunk HF_ (0 .. n_halves - 1) of the K range: chunk cc_begin + HF_ / 2, K-steps 2 * (HF_ & 1) ..
#define HS_WBASE(HF_) (wf0 + ((size_t)(cc_begin + ((HF_) >> 1)) * 36 + 2 * ((HF_) & 1)) * 64)
#define HS_PBASE(HF_) (wp0 + ((size_t)(cc_begin + ((HF_) >> 1)) * 4 + 2 * ((HF_) & 1)) * 64)
  u32x4 fa[3][2], fp2[2];
#define HS_LOAD_A(S_, BASE_, T_)                                                               \
  {                                                                                            \
    fa[S_][0] = (BASE_)[(T_) * 4 * 64];                                                        \
    fa[S_][1] = (BASE_)[(T_) * 4 * 64 + 64];                                                   \
  }

  const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  floatx16 acc[2] = {zero16, zero16}, acc2[2] = {zero16, zero16};

  // K-step Q_ (literal) of the current item: Q_ / 2 = tap (9: the projection, on the centre
  // tap's pixels), Q_ & 1 = which 16 of the item's 32 channels.  Pixel fragments are read BD
  // steps ahead (ring of BD + 1); weight stage tap % 3 is refilled behind its last use with
  // the tap three ahead, from the next item's block once that runs past this item's ninth tap.
  constexpr int BD = 3;
  half8 bf[BD + 1][2];
#define HS_TAPQ(Q_) ((Q_) / 2 == 9 ? 4 : (Q_) / 2)     /* the projection reads the centre tap */
#define HS_READ_B(Q_)                                                                          \
  {                                                                                            \
    const f16* fp_ = &s_patch[pb][((((HS_TAPQ(Q_) / 3) & 1) * 2 + ((HS_TAPQ(Q_) % 3) & 1)) * PLANE) * 32 + \
                                  fb[(HS_TAPQ(Q_) / 3) >> 1][(HS_TAPQ(Q_) % 3) >> 1][(Q_) & 1]]; \
    bf[(Q_) % (BD + 1)][0] = *reinterpret_cast<const half8*>(fp_);                             \
    bf[(Q_) % (BD + 1)][1] = *reinterpret_cast<const half8*>(fp_ + GOFF);                      \
  }
#define HS_KSTEP(Q_)                                                                           \
  {                                                                                            \
    if ((Q_) + BD < 20) { if ((Q_) + BD < 18 || has_proj) HS_READ_B((Q_) + BD) }               \
    if (((Q_) & 1) == 0 && more) {                                                             \
      if ((Q_) / 2 >= 3 && (Q_) / 2 - 3 < PL) HS_HAND_P((Q_) / 2 - 3, pb ^ 1)                  \
      if ((Q_) / 2 < PL) HS_LOAD_P((Q_) / 2)                                                   \
    }                                                                                          \
    if ((Q_) < 18) {                                                                           \
      const half8 a_ = __builtin_bit_cast(half8, fa[((Q_) / 2) % 3][(Q_) & 1]);                \
      _Pragma("unroll") for (int g = 0; g < 2; ++g)                                            \
        acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a_, bf[(Q_) % (BD + 1)][g], acc[g], 0, 0, 0); \
      if ((Q_) & 1) {                                                                          \
        if ((Q_) / 2 + 3 < 9) HS_LOAD_A(((Q_) / 2) % 3, w_cur, (Q_) / 2 + 3)                   \
        else HS_LOAD_A(((Q_) / 2) % 3, w_nxt, (Q_) / 2 + 3 - 9)                                \
      }                                                                                        \
    } else if (has_proj) {                                                                     \
      const half8 a_ = __builtin_bit_cast(half8, fp2[(Q_) & 1]);                               \
      _Pragma("unroll") for (int g = 0; g < 2; ++g)                                            \
        acc2[g] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a_, bf[(Q_) % (BD + 1)][g], acc2[g], 0, 0, 0); \
    }                                                                                          \
    __builtin_amdgcn_sched_barrier(0);                                                         \
  }

  // ---- prologue: first item's patch into buffer 0, its first three taps of weights
  int img, y0, x0;
  HS_TILE_SETUP(tm_begin, img, y0, x0)
  int pb = 0;
  {
    u32x4 first[PL];
    const int ch0 = cc_begin * 64;
#pragma unroll
    for (int i = 0; i < PL; ++i)
      first[i] = *reinterpret_cast<const u32x4*>(p.in + (l_poff[i] >= 0 ? l_poff[i] + ch0 : 0));
    const u32x4* w0 = HS_WBASE(0);
    HS_LOAD_A(0, w0, 0) HS_LOAD_A(1, w0, 1) HS_LOAD_A(2, w0, 2)
#pragma unroll
    for (int i = 0; i < PL; ++i)
      if (l_plds[i] >= 0) {
        const u32x4 zero = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4*>(&s_patch[0][l_plds[i]]) = l_poff[i] >= 0 ? first[i] : zero;
      }
  }
  __syncthreads();

  const int n_base = n0 + wave * 32 + h * 4;
  int tm = tm_begin, hf = 0;
  for (int item = 0; item < n_items; ++item) {
    // the item after this one: next half chunk of the tile, or the first of the next tile
    const bool more = item + 1 < n_items;
    const bool cross = hf + 1 == n_halves;
    const int hf_n = more ? (cross ? 0 : hf + 1) : hf;
    const int s_img = img, s_y0 = y0, s_x0 = x0;      // this item's tile (for the store below)
    if (more && cross) HS_TILE_SETUP(tm + 1, img, y0, x0)   // l_poff now describes the next tile
    const int ch_n = (cc_begin + (hf_n >> 1)) * 64 + (hf_n & 1) * 32;
    const u32x4* const w_cur = HS_WBASE(hf);
    const u32x4* const w_nxt = HS_WBASE(hf_n);
    if (has_proj) {
      const u32x4* pbase = HS_PBASE(hf);
      fp2[0] = pbase[0];
      fp2[1] = pbase[64];
    }
    HS_READ_B(0) HS_READ_B(1) HS_READ_B(2)
    HS_KSTEP(0) HS_KSTEP(1) HS_KSTEP(2) HS_KSTEP(3) HS_KSTEP(4) HS_KSTEP(5) HS_KSTEP(6)
    HS_KSTEP(7) HS_KSTEP(8) HS_KSTEP(9) HS_KSTEP(10) HS_KSTEP(11) HS_KSTEP(12) HS_KSTEP(13)
    HS_KSTEP(14) HS_KSTEP(15) HS_KSTEP(16) HS_KSTEP(17) HS_KSTEP(18) HS_KSTEP(19)
    if (cross) {
      // ---- the tile is complete: accumulator quad i of group g = channels n_base + 8*i .. +3 of
      // pixel (4*g + r/8, r%8) of the tile
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        const int oy = s_y0 + 4 * g + oy_l, ox = s_x0 + ox_l;
        const bool valid = oy < p.hout && ox < p.wout;
        const int m = s_img * p.img_m + oy * p.wout + ox;
        if (p.use_partial) {
          if (valid) {
            float* dst = p.partial + ((size_t)split * p.m + m) * p.cout_pad + n_base;
#pragma unroll
            for (int i = 0; i < 4; ++i)
              *reinterpret_cast<float4*>(dst + 8 * i) = make_float4(
                  acc[g][4 * i], acc[g][4 * i + 1], acc[g][4 * i + 2], acc[g][4 * i + 3]);
            if (has_proj) {
              float* dst2 = p.partial2 + ((size_t)split * p.m + m) * p.cout_pad + n_base;
#pragma unroll
              for (int i = 0; i < 4; ++i)
                *reinterpret_cast<float4*>(dst2 + 8 * i) = make_float4(
                    acc2[g][4 * i], acc2[g][4 * i + 1], acc2[g][4 * i + 2], acc2[g][4 * i + 3]);
            }
          }
        } else {
          // fp16 outputs with whole 128-channel tiles (the host selects this kernel only then)
          const half4 none[4] = {};
          store_octets(p, valid, m, n0 + wave * 32, h, acc[g], none, false);
          if (has_proj)                            // projection: no residual, no ReLU
            store_octets_to(p.out2, p.out2_pitch, false, valid, m, n0 + wave * 32, h, acc2[g], none,
                            false);
        }
      }
      acc[0] = acc[1] = zero16;
      acc2[0] = acc2[1] = zero16;
      ++tm;
    }
    hf = hf_n;
    __syncthreads();      // the next patch is complete, and every wavefront is done with this one
    pb ^= 1;
  }
#undef HS_KSTEP
#undef HS_READ_B
#undef HS_TAPQ
#undef HS_LOAD_A
#undef HS_PBASE
#undef HS_WBASE
#undef HS_HAND_P
#undef HS_LOAD_P
#undef HS_TILE_SETUP
}

constexpr int OCC3 = 2, OCC4 = 2;   // waves per SIMD the tile-walking instantiations are built for
KernelDesc describe(const ConvParams& p) {
  // 1-D grid, padded to a multiple of 8 so that every XCD owns tiles_per_xcd consecutive tiles
  const dim3 grid(8u * (unsigned)p.tiles_per_xcd);
  const bool walk = p.tiles_per_wg > 1;
  if (p.variant == 5) return KernelDesc{(const void*)k_block64_fused, grid, dim3(256), 0};
  if (p.variant == 6) return KernelDesc{(const void*)k_conv3x3_dira, grid, dim3(256), 0};
  if (p.variant == 7) return KernelDesc{(const void*)k_conv3x3s2_dira, grid, dim3(256), 0};
  if (p.variant == 1) return KernelDesc{(const void*)k_conv3x3_halo<1, 2, 9, 1, false, 1>, grid, dim3(256), 0};
  if (p.variant == 2) return KernelDesc{(const void*)k_conv3x3_halo<2, 2, 9, 1, false, 1>, grid, dim3(256), 0};
  if (p.variant == 3 && walk && p.chunks_per_tap == 1 && !p.use_partial && p.nsplit == 1 &&
      !p.out_f32 && p.cout % 64 == 0)
    return KernelDesc{(const void*)k_conv3x3_c64_walk, grid, dim3(256), 0};
  if (p.variant == 3 && walk && p.chunks_per_tap == 1)
    return KernelDesc{(const void*)k_conv3x3_halo<2, 1, 9, 1, true, OCC3>, grid, dim3(256), 0};
  if (p.variant == 3)
    return KernelDesc{walk ? (const void*)k_conv3x3_halo<2, 1, 3, 1, true, OCC3>
                           : (const void*)k_conv3x3_halo<2, 1, 3, 1, false, 1>, grid, dim3(256), 0};
  if (p.variant == 4)
    return KernelDesc{walk ? (const void*)k_conv3x3_halo<1, 1, 3, 2, true, OCC4>
                           : (const void*)k_conv3x3_halo<1, 1, 3, 2, false, 1>, grid, dim3(256), 0};
  const void* f = p.kc == 16   ? (const void*)k_conv_mfma<16, 4>
                  : p.kc == 32 ? (const void*)k_conv_mfma<32, 4>
                  : p.depth == 8 ? (const void*)k_conv_mfma<64, 8>
                               : (const void*)k_conv_mfma<64, 4>;
  return KernelDesc{f, grid, dim3(256), 0};
}

// ---------------------------------------------------------------------------------------------
// Split-K epilogue: one thread per (pixel, 4 channels).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_splitk_epilogue(SplitKEpilogueParams p) {
  const int quads = p.cout >> 2;
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)p.m * quads) return;
  const int m = (int)(t / quads), n = (int)(t - (size_t)m * quads) * 4;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int sidx = 0; sidx < p.nsplit; ++sidx) {
    const float4 v =
        *reinterpret_cast<const float4*>(p.partial + ((size_t)sidx * p.m + m) * p.cout_pad + n);
    a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
  }
  float v[4] = {a.x, a.y, a.z, a.w};
  if (p.res) {
    const half4 r = *reinterpret_cast<const half4*>(p.res + (size_t)m * p.res_pitch + n);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] += (float)r[j];
  }
  if (p.relu) {
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = fmaxf(v[j], 0.0f);
  }
  if (p.out_f32) {
    const int b = m / p.img_m, ml = m - b * p.img_m;
#pragma unroll
    for (int j = 0; j < 4; ++j) p.out_f32[((size_t)b * p.cout + n + j) * p.img_m + ml] = v[j];
  } else {
    half4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (f16)v[j];
    *reinterpret_cast<half4*>(p.out + (size_t)m * p.out_pitch + n) = o;
  }
  if (p.partial2) {
    float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int sidx = 0; sidx < p.nsplit; ++sidx) {
      const float4 v2 = *reinterpret_cast<const float4*>(
          p.partial2 + ((size_t)sidx * p.m + m) * p.cout_pad + n);
      b.x += v2.x; b.y += v2.y; b.z += v2.z; b.w += v2.w;
    }
    half4 o2;
    o2[0] = (f16)b.x; o2[1] = (f16)b.y; o2[2] = (f16)b.z; o2[3] = (f16)b.w;
    *reinterpret_cast<half4*>(p.out2 + (size_t)m * p.out2_pitch + n) = o2;
  }
}

KernelDesc describe(const SplitKEpilogueParams& p) {
  const size_t n = (size_t)p.m * (p.cout >> 2);
  return KernelDesc{(const void*)k_splitk_epilogue, dim3((unsigned)((n + 255) / 256)), dim3(256), 0};
}

// ---------------------------------------------------------------------------------------------
// ConvLSTM epilogue + 1x1 head: one workgroup per pixel, one thread per hidden channel
// (hid == 256).  Gates and state update in fp32 (c kept in fp32, h stored fp16); the head's
// eight logits of the pixel are the workgroup-wide sums of w[k][j] * h[j] over the stored
// (fp16) h: a wavefront butterfly, then the four wavefront sums in order.
// logits: planar per image, logits[(image*8 + k)*img_m + pixel in image].
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_lstm_epilogue(LstmEpilogueParams p) {
  __shared__ float s_part[4][8];
  const int m = blockIdx.x, j = threadIdx.x, lane = j & 63, wave = j >> 6;
  const size_t t = (size_t)m * p.hid + j;
  const int n4 = 4 * p.hid;
  float g[4] = {0.f, 0.f, 0.f, 0.f};
  for (int sidx = 0; sidx < p.nsplit; ++sidx) {
    const float* row = p.partial + ((size_t)sidx * p.m + m) * n4;
#pragma unroll
    for (int k = 0; k < 4; ++k) g[k] += row[k * p.hid + j];
  }
  const float gi = sigmoid_f(g[0]), gf = sigmoid_f(g[1]), gg = tanhf(g[2]), go = sigmoid_f(g[3]);
  const float c_new = gf * p.c[t] + gi * gg;
  p.c[t] = c_new;
  const f16 h16 = (f16)(go * tanhf(c_new));
  p.h_out[(size_t)m * p.h_pitch + j] = h16;

  const float hv = (float)h16;
  float v[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) v[k] = hv * (float)p.w_head[k * p.hid + j];
  // Wavefront sums of the eight products by a halving butterfly: at offset 32 a lane keeps four
  // of the eight (k / 4 == its bit 5) and hands the other four to its partner in the same
  // exchange, at 16 two, at 8 one; offsets 4, 2, 1 finish that one.  Ten exchanges instead of
  // 48, and every sum adds the same pairs level by level as the full butterfly would: lanes
  // 8 * k .. 8 * k + 7 end with the sum of product k.
  float a4[4], a2[2], a1;
  {
    const bool up = (lane & 32) != 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      a4[i] = (up ? v[4 + i] : v[i]) + __shfl_xor(up ? v[i] : v[4 + i], 32, 64);
  }
  {
    const bool up = (lane & 16) != 0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
      a2[i] = (up ? a4[2 + i] : a4[i]) + __shfl_xor(up ? a4[i] : a4[2 + i], 16, 64);
  }
  {
    const bool up = (lane & 8) != 0;
    a1 = (up ? a2[1] : a2[0]) + __shfl_xor(up ? a2[0] : a2[1], 8, 64);
  }
#pragma unroll
  for (int off = 4; off >= 1; off >>= 1) a1 += __shfl_xor(a1, off, 64);
  if ((lane & 7) == 0) s_part[wave][lane >> 3] = a1;
  __syncthreads();
  if (j < 8) {
    const float sum = ((s_part[0][j] + s_part[1][j]) + s_part[2][j]) + s_part[3][j];
    const int img = m / p.img_m, ml = m - img * p.img_m;
    p.logits[((size_t)img * 8 + j) * p.img_m + ml] = sum;
  }
}

KernelDesc describe(const LstmEpilogueParams& p) {
  return KernelDesc{(const void*)k_lstm_epilogue, dim3((unsigned)p.m), dim3(256), 0};
}

// =============================================================================================
// Stem: 7x7 stride-2 convolution (3 -> 64 channels) + ReLU + 3x3 stride-2 max-pool in one
// kernel; the 64-channel convolution output (the largest tensor of the network) never reaches
// memory.
//
// A workgroup produces 8 x 15 pooled pixels, i.e. the 17 x 31 convolution outputs under them
// (one row/column of overlap with the neighbouring tiles), as 17 row fragments of 32 pixels.
// The whole input patch (39 rows x 70 padded 4-channel pixels) sits in LDS; the weight matrix
// (64 x 224 halves, k = (ky*8 + px)*4 + ch) is held as MFMA fragments in registers.  Because the image is stored with 4
// channels per pixel, the 32 K-values of kernel row ky for convolution pixel cx are the 64
// contiguous bytes starting at input pixel 2*cx of row 2*cy + ky: MFMA pixel operands are read
// straight from the patch, no im2col copy.
// Wavefront (wm, wn): convolution rows 8*wm .. 8*wm+8 (row 8 is computed by both halves, it
// feeds pooled rows 3 and 4), channels 32*wn .. +31: nine accumulators.  Pooling: maximum over
// three accumulators (rows), then over lanes r, r+1, r+2 (columns, two DPP wavefront shifts),
// ReLU last; even lanes store.
// Rounding to fp16 after the maximum equals the maximum of the rounded values.
// =============================================================================================
// value of lane + 1 (DPP whole-wavefront shift; lane 63 keeps its own)
__device__ __forceinline__ float lane_plus_1(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), 0x130,
                                                    0xf, 0xf, false));
}

__global__ __launch_bounds__(256, 2) void k_stem_pool(StemPoolParams p) {
  constexpr int PROWS = 39, PVEC = 35, PROW_H = PVEC * 8;      // patch rows, vectors, halves per row
  constexpr int NPV = PROWS * PVEC, NPL = (NPV + 255) / 256;   // patch vectors, per thread
  __shared__ __align__(16) f16 s_patch[PROWS * PROW_H];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, h = lane >> 5;
  const int tile = (int)(blockIdx.x & 7u) * p.tiles_per_xcd + (int)(blockIdx.x >> 3);
  if (tile >= p.batch * p.tiles_y * p.tiles_x) return;
  const int tx = tile % p.tiles_x, ty = (tile / p.tiles_x) % p.tiles_y;
  const int img = tile / (p.tiles_x * p.tiles_y);
  const int p0 = 8 * ty, q0 = 15 * tx;              // first pooled pixel
  const int cy0 = 2 * p0 - 1, cx0 = 2 * q0 - 1;     // first convolution pixel
  const int iy0 = 2 * cy0, ix0 = 2 * cx0;           // first pixel of the padded image (may be < 0)

  // ---- fill LDS: unconditional loads from clamped addresses, zeros where out of the image
  u32x4 st_p[NPL];
  bool inb[NPL];
#pragma unroll
  for (int i = 0; i < NPL; ++i) {
    const int v = min(tid + 256 * i, NPV - 1);
    const int ly = v / PVEC, lv = v - ly * PVEC;
    const int y = iy0 + ly, x = ix0 + 2 * lv;
    inb[i] = y >= 0 && y < p.hin && x >= 0 && x < p.win;
    const f16* src = inb[i] ? p.in + (((size_t)img * p.hin + y) * p.win + x) * 4 : p.in;
    st_p[i] = *reinterpret_cast<const u32x4*>(src);
  }
  // The wavefront's 14 weight fragments come straight from memory (fragment order, one
  // contiguous 1 KB block per wavefront load) and stay in registers.
  const int wm = wave & 1, wn = wave >> 1;
  half8 a[7][2];
  {
    const half8* wfr = reinterpret_cast<const half8*>(p.wt) + (size_t)wn * 14 * 64 + lane;
#pragma unroll
    for (int ky = 0; ky < 7; ++ky)
#pragma unroll
      for (int s = 0; s < 2; ++s) a[ky][s] = wfr[(ky * 2 + s) * 64];
  }
#pragma unroll
  for (int i = 0; i < NPL; ++i) {
    const int v = tid + 256 * i;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    if (v < NPV) *reinterpret_cast<u32x4*>(&s_patch[v * 8]) = inb[i] ? st_p[i] : zero;
  }
  __syncthreads();

  // ---- 14 K-steps of 16 (two per kernel row), nine row fragments each
  floatx16 acc[9];
#pragma unroll
  for (int j = 0; j < 9; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.0f;
  const f16* fp = &s_patch[(16 * wm) * PROW_H + r * 8 + h * 8];   // patch row 2*(8*wm + j) + ky
  // Patch row rho serves every (convolution row j, kernel row ky) with 2*j + ky == rho, so each
  // patch fragment is read once: 46 LDS reads feed the 126 MFMAs.  Per accumulator the K order
  // stays ky = 0..6.
#pragma unroll
  for (int rho = 0; rho < 23; ++rho) {
    if (rho % 4 == 3) __builtin_amdgcn_sched_barrier(0);   // bounds how far reads are hoisted
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const half8 b = *reinterpret_cast<const half8*>(fp + rho * PROW_H + s * 16);
#pragma unroll
      for (int j = 0; j < 9; ++j) {
        const int ky = rho - 2 * j;
        if (ky >= 0 && ky <= 6)
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[ky < 0 ? 0 : ky > 6 ? 6 : ky][s], b,
                                                         acc[j], 0, 0, 0);
      }
    }
  }

  // ---- pool, ReLU.  max and ReLU commute, so ReLU comes last; a pooling window always holds
  // its centre row (convolution row 2 * py exists whenever pooled row py does), rows outside the
  // convolution output are skipped (the same for the whole wavefront), columns outside it count
  // as 0, which cannot change ReLU(max).  Then the lane pair (r, r + 32) exchanges quads and
  // stores 16 bytes per lane (store_octets_to); every lane takes part in the exchange.
  const int cx = cx0 + r;
  const bool col_ok = cx >= 0 && cx < p.wc;
  const int q = q0 + (r >> 1);
  const bool writer = (r & 1) == 0 && r <= 28 && q < p.wp;
#pragma unroll
  for (int pl = 0; pl < 4; ++pl) {
    const int py = p0 + 4 * wm + pl;
    const int cy_top = cy0 + 8 * wm + 2 * pl;             // rows cy_top, cy_top + 1 (centre), cy_top + 2
    const bool top_ok = cy_top >= 0, bot_ok = cy_top + 2 < p.hc;
    floatx16 v = acc[2 * pl + 1];
    if (top_ok) {
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = fmaxf(v[i], acc[2 * pl][i]);
    }
    if (bot_ok) {
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = fmaxf(v[i], acc[2 * pl + 2][i]);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float m = col_ok ? v[i] : 0.0f;
      const float m2 = fmaxf(m, lane_plus_1(m));       // columns r, r+1
      v[i] = fmaxf(fmaxf(m2, lane_plus_1(m2)), 0.0f);  // columns r .. r+2, ReLU
    }
    const half4 none[4] = {};
    store_octets_to(p.out, 64, false, writer && py < p.hp, (img * p.hp + py) * p.wp + q, 32 * wn, h, v,
                    none, false);
  }
}

KernelDesc describe(const StemPoolParams& p) {
  return KernelDesc{(const void*)k_stem_pool, dim3(8u * (unsigned)p.tiles_per_xcd), dim3(256), 0};
}

// =============================================================================================
// Stage 3: one workgroup per tool channel (plus one for the overlay's channel map).  Every lane keeps (best value, lowest index);
// wavefront butterfly reduction, then one more across the 4 wavefronts through LDS.
// The integer outputs are decided on the logits with exact comparisons.
// =============================================================================================
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) {
  return v > bv || (v == bv && i < bi);
}

__global__ __launch_bounds__(256) void k_postprocess(PostParams p) {
  __shared__ float s_v[4];
  __shared__ int s_i[4];
  const int k = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t img_off = (size_t)blockIdx.y * 8 * p.n;   // image blockIdx.y of the batch
  if (k == 8) {
    // ninth workgroup: per cell the lowest channel whose mask is set (what the overlay draws),
    // decided on the logits with the same comparison as the masks
    for (int i = tid; i < p.n; i += 256) {
      uint8_t lowest = 0xff;
#pragma unroll
      for (int c = 7; c >= 0; --c)
        if (p.logits[img_off + (size_t)c * p.n + i] > p.theta) lowest = (uint8_t)c;
      p.kmap[(size_t)blockIdx.y * p.n + i] = lowest;
    }
    return;
  }
  float* const heat = p.heat + img_off;
  uint8_t* const mask = p.mask + img_off;
  PostRecord* const rec = p.rec + blockIdx.y;
  const float* L = p.logits + img_off + (size_t)k * p.n;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = tid; i < p.n; i += 256) {
    const float x = L[i];
    heat[(size_t)k * p.n + i] = 1.0f / (1.0f + expf(-x));
    mask[(size_t)k * p.n + i] = x > p.theta ? 1 : 0;
    if (better(x, i, bv, bi)) { bv = x; bi = i; }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(bv, off, 64);
    const int oi = __shfl_xor(bi, off, 64);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
  }
  if (lane == 0) { s_v[wave] = bv; s_i[wave] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 4; ++w)
      if (better(s_v[w], s_i[w], bv, bi)) { bv = s_v[w]; bi = s_i[w]; }
    rec->argmax_idx[k] = bi;
    rec->peak[k] = 1.0f / (1.0f + expf(-bv));
    rec->present[k] = bv > p.theta ? 1 : 0;
    if (p.marks) {
      // anchor of the annotation layer: centre of the argmax cell's footprint in the frame
      int* mk = p.marks + ((size_t)blockIdx.y * 8 + k) * 2;
      if (bv > p.theta) {
        const int ay = bi / p.wm, ax = bi - ay * p.wm;
        mk[0] = ((2 * ax + 1) * p.wf) / (2 * p.wm);
        mk[1] = ((2 * ay + 1) * p.hf) / (2 * p.hm);
      } else {
        mk[0] = -1;
        mk[1] = -1;
      }
    }
  }
}

KernelDesc describe(const PostParams& p) {
  return KernelDesc{(const void*)k_postprocess, dim3(9, p.batch), dim3(256), 0};
}

// =============================================================================================
// Stage 4: pure streaming.  A thread owns one group of 16 pixels (48 bytes, three 16-byte
// accesses) of one frame row; groups are numbered row-major over the frame, 256 per workgroup,
// so there is no per-row prologue and no barrier.  A group spans at most two cells of the
// channel map when a cell is at least 16 pixels wide: both are fetched up front together with
// the pixels (a third cell, on tiny frames, is fetched on demand).  Where the frame rows are
// contiguous, a wavefront moves its 3072 bytes as fully coalesced 16-byte vectors and regroups
// them through LDS, instead of every lane touching its own 48-byte span.
// =============================================================================================
// One layer of stage 4 applied to a group of 16 pixels held in registers (w[0..11], word j starts
// with channel j mod 3): blend of the layer's channel map, then its annotations.
// Colour of channel k (0..7).  A select chain over the eight scalar palette words: indexing the
// kernel-argument array with a per-lane k would be a vector load from memory, one more full
// memory latency between the channel byte and the blend.
__device__ __forceinline__ uint32_t overlay_colour(const OverlayLayer& L, uint32_t k) {
  uint32_t c = L.pal[0];
#pragma unroll
  for (uint32_t i = 1; i < 8; ++i) c = k == i ? L.pal[i] : c;
  return c;
}

// The channel-map cells a group of 16 pixels starting at (X0, Y) can see in layer L: its first
// cell, and the two channel bytes fetched up front (a third cell, on tiny frames, on demand).
struct OverlayCells {
  const uint8_t* krow;
  int mx0;
  uint8_t k0, k1;
};
__device__ __forceinline__ OverlayCells overlay_cells(const OverlayParams& p, const OverlayLayer& L,
                                                      int Y, int X0, int by) {
  OverlayCells c;
  const int my = (int)udiv_est((uint32_t)(Y * L.hm), (uint32_t)p.hf, p.rcp_hf);
  c.krow = L.kmap + ((size_t)by * L.hm + my) * L.wm;
  c.mx0 = (int)udiv_est((uint32_t)(X0 * L.wm), (uint32_t)p.wf, p.rcp_wf);
  c.k0 = c.krow[c.mx0];
  c.k1 = c.krow[min(c.mx0 + 1, L.wm - 1)];
  return c;
}

__device__ __forceinline__ void overlay_layer_group(const OverlayParams& p, const OverlayLayer& L,
                                                    const OverlayCells& cells, uint32_t (&w)[12],
                                                    int Y, int X0, int by) {
  const uint8_t* krow = cells.krow;
  const int ia = 256 - L.a;
  const int mx0 = cells.mx0;
  const uint8_t k0 = cells.k0, k1 = cells.k1;
  // Most groups see one channel for all 16 pixels: nothing to draw, or one colour.  Then the
  // blend runs on two bytes per 32-bit operation: even and odd bytes of a word are 16-bit
  // fields, (256 - a) * byte + (a * colour + 128) never exceeds 65408, so no field carries into
  // its neighbour.  The field pair is below 2^24 and the factor at most 256: 24-bit multiplies
  // (full rate; the 32-bit ones run at a quarter of it) are exact.
  const int mx_last = (int)udiv_est((uint32_t)((X0 + 15) * L.wm), (uint32_t)p.wf, p.rcp_wf);
  const bool one_cell = mx_last == mx0 || (mx_last == mx0 + 1 && k1 == k0);
  if (one_cell) {
    if (k0 != 0xff) {
      const uint32_t col = overlay_colour(L, k0);
      uint32_t t[3];
#pragma unroll
      for (int c = 0; c < 3; ++c) t[c] = mad24((uint32_t)L.a, (col >> (8 * c)) & 0xffu, 128u);
#pragma unroll
      for (int j = 0; j < 12; ++j) {
        const uint32_t ce = t[j % 3] | (t[(j + 2) % 3] << 16);        // bytes 0 and 2
        const uint32_t co = t[(j + 1) % 3] | (t[(j + 3) % 3] << 16);  // bytes 1 and 3
        const uint32_t e = w[j] & 0x00ff00ffu, o = (w[j] >> 8) & 0x00ff00ffu;
        w[j] = ((mad24(e, (uint32_t)ia, ce) >> 8) & 0x00ff00ffu) |
               (mad24(o, (uint32_t)ia, co) & 0xff00ff00u);
      }
    }
  } else if (mx_last == mx0 + 1) {
    // two cells: pixels [0, s) see k0, [s, 16) see k1.  Same packed blend with the colour
    // term chosen per byte (byte index < 3*s), then bytes of an undrawn cell are restored.
    const int rem = X0 * L.wm - mx0 * p.wf;
    const int s3 = 3 * (int)udiv_est((uint32_t)(p.wf - rem + L.wm - 1), (uint32_t)L.wm, L.rcp_wm);
    const uint32_t c0 = k0 != 0xff ? overlay_colour(L, k0) : 0u;
    const uint32_t c1 = k1 != 0xff ? overlay_colour(L, k1) : 0u;
    const uint32_t d0 = k0 != 0xff ? 0xffffffffu : 0u, d1 = k1 != 0xff ? 0xffffffffu : 0u;
    uint32_t t0[3], t1[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      t0[c] = mad24((uint32_t)L.a, (c0 >> (8 * c)) & 0xffu, 128u);
      t1[c] = mad24((uint32_t)L.a, (c1 >> (8 * c)) & 0xffu, 128u);
    }
#pragma unroll
    for (int j = 0; j < 12; ++j) {
      const uint32_t tb0 = 4 * j + 0 < s3 ? t0[j % 3] : t1[j % 3];
      const uint32_t tb1 = 4 * j + 1 < s3 ? t0[(j + 1) % 3] : t1[(j + 1) % 3];
      const uint32_t tb2 = 4 * j + 2 < s3 ? t0[(j + 2) % 3] : t1[(j + 2) % 3];
      const uint32_t tb3 = 4 * j + 3 < s3 ? t0[(j + 3) % 3] : t1[(j + 3) % 3];
      const uint32_t e = w[j] & 0x00ff00ffu, o = (w[j] >> 8) & 0x00ff00ffu;
      const uint32_t blended = ((mad24(e, (uint32_t)ia, tb0 | (tb2 << 16)) >> 8) & 0x00ff00ffu) |
                               (mad24(o, (uint32_t)ia, tb1 | (tb3 << 16)) & 0xff00ff00u);
      const int nb = min(4, max(0, s3 - 4 * j));                    // leading bytes of cell 0
      const uint32_t low = nb == 4 ? 0xffffffffu : ((1u << (8 * nb)) - 1u);
      const uint32_t draw = (low & d0) | (~low & d1);
      w[j] = (blended & draw) | (w[j] & ~draw);
    }
  } else {
    int mx = mx0;
    int rem = X0 * L.wm - mx0 * p.wf;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint8_t k = mx == mx0 ? k0 : (mx == mx0 + 1 ? k1 : krow[mx]);
      if (k != 0xff) {
        const uint32_t col = overlay_colour(L, k);
#pragma unroll
        for (int c = 0; c < 3; ++c) {
          const int byte = 3 * i + c;                 // literal after unrolling
          const uint32_t pc = (col >> (8 * c)) & 0xffu;
          const uint32_t old = (w[byte >> 2] >> (8 * (byte & 3))) & 0xffu;
          const uint32_t nw = mad24((uint32_t)L.a, pc, mad24((uint32_t)ia, old, 128u)) >> 8;
          w[byte >> 2] = (w[byte >> 2] & ~(0xffu << (8 * (byte & 3)))) | (nw << (8 * (byte & 3)));
        }
      }
      rem += L.wm;
      while (rem >= p.wf) { rem -= p.wf; ++mx; }
    }
  }
  if (L.marks) {
    // annotation layer: a tool's drawing lies in one box; only groups that meet a box look
    // closer, pixel by pixel, tools in increasing order (later tools paint over earlier ones)
    const int* mk = L.marks + (size_t)by * 16;
    const int lab_w = 11 * L.scale, lab_h = 7 * L.scale;
#pragma unroll 1
    for (int k = 0; k < 8; ++k) {
      const int cx = mk[2 * k], cy = mk[2 * k + 1];
      if (cx < 0) continue;
      const int ox = cx + L.arm + 2, oy = cy - lab_h - 2;          // label origin
      if (Y < min(cy - L.arm, oy) || Y > cy + L.arm || X0 + 15 < cx - L.arm || X0 >= ox + lab_w)
        continue;
      const uint32_t col = L.pal[k];
      // what this row paints, as pixel intervals around cx and a bit per label pixel
      const int dy = abs(Y - cy);
      const int reach = dy <= L.half ? L.arm : (dy <= L.arm ? L.half : -1);   // |X - cx| <= reach
      uint64_t lab_lo = 0, lab_hi = 0;       // label pixels lx = 0..63 and 64..87 of this row
      if (Y >= oy && Y < oy + lab_h) {
        const int gy = (int)udiv_est((uint32_t)(Y - oy), (uint32_t)L.scale, L.rcp_scale);
        const uint32_t cells = (uint32_t)((L.glyph[0] >> (5 * gy)) & 31ull) |
                               ((uint32_t)((L.glyph[1 + k] >> (5 * gy)) & 31ull) << 6);
        const uint64_t run = (1ull << L.scale) - 1ull;               // scale <= 8 pixels per cell
        for (int cell = 0; cell < 11; ++cell) {
          if (!((cells >> cell) & 1u)) continue;
          const int at = cell * L.scale;
          if (at < 64) lab_lo |= run << at;
          if (at + L.scale > 64) lab_hi |= at >= 64 ? run << (at - 64) : run >> (64 - at);
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int X = X0 + i, lx = X - ox;
        bool hit = abs(X - cx) <= reach;
        if (lx >= 0 && lx < lab_w) hit = hit || (((lx < 64 ? lab_lo >> lx : lab_hi >> (lx - 64)) & 1ull) != 0);
        if (hit) {
#pragma unroll
          for (int c = 0; c < 3; ++c) {
            const int byte = 3 * i + c;               // literal after unrolling
            const uint32_t pc = (col >> (8 * c)) & 0xffu;
            w[byte >> 2] = (w[byte >> 2] & ~(0xffu << (8 * (byte & 3)))) | (pc << (8 * (byte & 3)));
          }
        }
      }
    }
  }
}

// The same layer applied to one pixel (x[0..2]) of a ragged row tail.
__device__ __forceinline__ void overlay_layer_pixel(const OverlayParams& p, const OverlayLayer& L,
                                                    uint32_t (&x)[3], int Y, int X, int by) {
  const int my = (int)udiv_est((uint32_t)(Y * L.hm), (uint32_t)p.hf, p.rcp_hf);
  const int mx = (int)udiv_est((uint32_t)(X * L.wm), (uint32_t)p.wf, p.rcp_wf);
  const uint8_t k = L.kmap[((size_t)by * L.hm + my) * L.wm + mx];
  int paint = -1;                          // tool whose marker or label covers this pixel
  if (L.marks) {
    const int* mk = L.marks + (size_t)by * 16;
    for (int t = 0; t < 8; ++t) {
      const int cx = mk[2 * t], cy = mk[2 * t + 1];
      if (cx < 0) continue;
      const int dx = abs(X - cx), dy = abs(Y - cy);
      bool hit = (dx <= L.arm && dy <= L.half) || (dy <= L.arm && dx <= L.half);
      const int lx = X - (cx + L.arm + 2), ly = Y - (cy - 7 * L.scale - 2);
      if (lx >= 0 && lx < 11 * L.scale && ly >= 0 && ly < 7 * L.scale) {
        const int cell = lx / L.scale, gy = ly / L.scale;
        const int gi = cell >= 6 ? 1 : 0, gx = cell - 6 * gi;
        if (gx < 5) hit = hit || ((L.glyph[gi ? 1 + t : 0] >> (5 * gy + gx)) & 1ull);
      }
      if (hit) paint = t;
    }
  }
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    if (k != 0xff) {
      const uint32_t pc = (overlay_colour(L, k) >> (8 * c)) & 0xffu;
      x[c] = mad24((uint32_t)L.a, pc, mad24((uint32_t)(256 - L.a), x[c], 128u)) >> 8;
    }
    if (paint >= 0) x[c] = (overlay_colour(L, (uint32_t)paint) >> (8 * c)) & 0xffu;
  }
}

// LAYERS == false: exactly one layer (every single-network application).  LAYERS == true: the
// n_layers layers of a multi-network application are applied in order, each on the result of
// the one before, while the pixels sit in registers (one read and one write of the frame).
template <bool LAYERS>
__global__ __launch_bounds__(256) void k_overlay(OverlayParams p) {
  __shared__ u32x4 s_x[4][192];
  const int gpr = (p.wf + 15) >> 4;                              // groups per row
  const int g = (int)blockIdx.x * 256 + (int)threadIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g_wave = g - lane;                                   // first group of the wavefront
  // rows of whole groups butt against each other and the wavefront is full (uniform per wavefront)
  const bool coalesced =
      (p.wf & 15) == 0 && p.pitch == (size_t)48 * gpr && g_wave + 64 <= gpr * p.hf;
  if (g >= gpr * p.hf) return;
  // all quotients by float estimate + exact fix-up (operands < 2^31, quotients < 2^22)
  const int Y = (int)udiv_est((uint32_t)g, (uint32_t)gpr, p.rcp_gpr), X0 = (g - Y * gpr) * 16;
  const uint8_t* srow = p.src[blockIdx.y] + (size_t)Y * p.pitch;
  uint8_t* drow = p.dst[blockIdx.y] + (size_t)Y * p.pitch;
  const int npx = min(16, p.wf - X0);
  const int nl = LAYERS ? p.n_layers : 1;
  if (npx == 16) {
    // the first layer's map bytes are requested before the pixels, so the two fetches overlap
    const OverlayCells first = overlay_cells(p, p.layer[0], Y, X0, (int)blockIdx.y);
    u32x4 v[3];
    if (coalesced) {
      // the wavefront's 64 groups are 3072 contiguous bytes: fetch them as 3 x 64 consecutive
      // 16-byte vectors and regroup through LDS (own region per wavefront, no workgroup barrier)
      const u32x4* s4 = reinterpret_cast<const u32x4*>(p.src[blockIdx.y] + (size_t)g_wave * 48);
      const u32x4 t0 = s4[lane], t1 = s4[64 + lane], t2 = s4[128 + lane];
      s_x[wave][lane] = t0; s_x[wave][64 + lane] = t1; s_x[wave][128 + lane] = t2;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      v[0] = s_x[wave][3 * lane]; v[1] = s_x[wave][3 * lane + 1]; v[2] = s_x[wave][3 * lane + 2];
    } else {
      const u32x4* s4 = reinterpret_cast<const u32x4*>(srow + (size_t)X0 * 3);
      v[0] = s4[0]; v[1] = s4[1]; v[2] = s4[2];
    }
    uint32_t w[12];
#pragma unroll
    for (int i = 0; i < 12; ++i) w[i] = v[i >> 2][i & 3];
    overlay_layer_group(p, p.layer[0], first, w, Y, X0, (int)blockIdx.y);
    if (LAYERS) {
#pragma unroll 1
      for (int l = 1; l < nl; ++l)
        overlay_layer_group(p, p.layer[l], overlay_cells(p, p.layer[l], Y, X0, (int)blockIdx.y), w,
                            Y, X0, (int)blockIdx.y);
    }
    if (coalesced) {
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        u32x4 o = {w[4 * j], w[4 * j + 1], w[4 * j + 2], w[4 * j + 3]};
        s_x[wave][3 * lane + j] = o;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      u32x4* d4 = reinterpret_cast<u32x4*>(p.dst[blockIdx.y] + (size_t)g_wave * 48);
      d4[lane] = s_x[wave][lane];
      d4[64 + lane] = s_x[wave][64 + lane];
      d4[128 + lane] = s_x[wave][128 + lane];
    } else {
      u32x4* d4 = reinterpret_cast<u32x4*>(drow + (size_t)X0 * 3);
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        u32x4 o = {w[4 * j], w[4 * j + 1], w[4 * j + 2], w[4 * j + 3]};
        d4[j] = o;
      }
    }
  } else {
    for (int i = 0; i < npx; ++i) {
      const int X = X0 + i;
      uint32_t x[3];
      for (int c = 0; c < 3; ++c) x[c] = srow[(size_t)X * 3 + c];
      for (int l = 0; l < nl; ++l) overlay_layer_pixel(p, p.layer[l], x, Y, X, (int)blockIdx.y);
      for (int c = 0; c < 3; ++c) drow[(size_t)X * 3 + c] = (uint8_t)x[c];
    }
  }
}

KernelDesc describe(const OverlayParams& p) {
  const unsigned groups = (unsigned)(((p.wf + 15) >> 4) * p.hf);
  const void* f = p.n_layers > 1 ? (const void*)k_overlay<true> : (const void*)k_overlay<false>;
  return KernelDesc{f, dim3((groups + 255) / 256, p.batch), dim3(256), 0};
}

// ---------------------------------------------------------------------------------------------
// Split-K scratch for callers that cannot allocate.  In host code the array's name is only a
// handle for hipGetSymbolAddress: every GPU holds its own copy at its own address, looked up
// once per device (with that device current) and used as an ordinary device pointer from then
// on -- the kernels receive it in their parameter blocks like the workspace scratch it replaces.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t static_scratch_address(void** d_ptr, size_t* bytes) {
  constexpr int kMaxDevices = 64;
  static void* ptr_of[kMaxDevices] = {nullptr};
  static std::mutex mu;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(mu);
  if (!ptr_of[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    ptr_of[dev] = ptr;
  }
  *d_ptr = ptr_of[dev];
  *bytes = kStaticScratchBytes;
  return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_fill_zero(uint4* d, size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride)
    d[i] = make_uint4(0, 0, 0, 0);
}

// Plain streaming copy (16-byte vectors, grid-stride): the known-size kernel that hardware
// byte counters are calibrated against.
__global__ __launch_bounds__(256) void k_copy(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                              size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

void launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 16;
  if (n == 0) return;
  const unsigned blocks = (unsigned)min((size_t)8192, (n + 255) / 256);
  hipLaunchKernelGGL(k_copy, dim3(blocks), dim3(256), 0, s, reinterpret_cast<const uint4*>(src),
                     reinterpret_cast<uint4*>(dst), n);
}

void launch_fill_zero(void* d, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 16;
  if (n == 0) return;
  const unsigned blocks = (unsigned)min((size_t)2048, (n + 255) / 256);
  hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, s, reinterpret_cast<uint4*>(d), n);
}

}  // namespace hs
