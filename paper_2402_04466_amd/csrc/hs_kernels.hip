// HIP kernels (gfx950 / CDNA4 only) of the per-frame tool-tracking hot path:
// paper Section III-A stages format conversion -> inference -> postprocess -> overlay.
#include "hs_kernels.h"

namespace hs {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

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
__global__ __launch_bounds__(256) void k_resize_norm(ResizeParams p) {
  extern __shared__ __align__(16) uint8_t lds[];
  __shared__ float s_lut32[256];
  __shared__ f16 s_lut16[256];
  const int tid = threadIdx.x;
  const int Y = blockIdx.x;
  const uint32_t dy = 2u * (uint32_t)p.ho, dx = 2u * (uint32_t)p.wo;
  int ny = (2 * Y + 1) * p.hi - p.ho;
  ny = max(0, min(ny, (p.hi - 1) * (int)dy));
  const uint32_t y0 = udiv_est((uint32_t)ny, dy, p.rcp_dy);
  const uint32_t fy = (uint32_t)ny - y0 * dy;
  const uint32_t y1 = min(y0 + 1u, (uint32_t)(p.hi - 1));

  const int row_vecs = (3 * p.wi + 15) >> 4;          // 16-byte vectors per source row
  const uint4* r0 = reinterpret_cast<const uint4*>(p.src + (size_t)y0 * p.src_pitch);
  const uint4* r1 = reinterpret_cast<const uint4*>(p.src + (size_t)y1 * p.src_pitch);
  uint4* l0 = reinterpret_cast<uint4*>(lds);
  uint4* l1 = l0 + row_vecs;
  for (int v = tid; v < row_vecs; v += 256) {
    l0[v] = r0[v];
    l1[v] = r1[v];
  }
  s_lut32[tid] = p.lut32[tid];
  s_lut16[tid] = p.lut16[tid];
  __syncthreads();

  const uint8_t* p0 = lds;
  const uint8_t* p1 = lds + (size_t)row_vecs * 16;
  const uint32_t d = dx * dy;
  const uint32_t wy1 = fy, wy0 = dy - fy;
  for (int X = tid; X < p.wo; X += 256) {
    int nx = (2 * X + 1) * p.wi - p.wo;
    nx = max(0, min(nx, (p.wi - 1) * (int)dx));
    const uint32_t x0 = udiv_est((uint32_t)nx, dx, p.rcp_dx);
    const uint32_t fx = (uint32_t)nx - x0 * dx;
    const uint32_t x1 = min(x0 + 1u, (uint32_t)(p.wi - 1));
    const uint32_t wx1 = fx, wx0 = dx - fx;
    uint32_t q[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      const uint32_t p00 = p0[3 * x0 + c], p01 = p0[3 * x1 + c];
      const uint32_t p10 = p1[3 * x0 + c], p11 = p1[3 * x1 + c];
      const uint32_t acc = wy0 * (wx0 * p00 + wx1 * p01) + wy1 * (wx0 * p10 + wx1 * p11);
      q[c] = udiv_est(acc + (d >> 1), d, p.rcp_d);
    }
    half4 px;
    px[0] = s_lut16[q[0]];
    px[1] = s_lut16[q[1]];
    px[2] = s_lut16[q[2]];
    px[3] = (f16)0.0f;
    *reinterpret_cast<half4*>(p.dst + ((size_t)(Y + p.pad_t) * p.dst_w + (X + p.pad_l)) * 4) = px;
    if (p.dst_f32) {
      const size_t plane = (size_t)p.ho * p.wo;
      float* o = p.dst_f32 + (size_t)Y * p.wo + X;
      o[0] = s_lut32[q[0]];
      o[plane] = s_lut32[q[1]];
      o[2 * plane] = s_lut32[q[2]];
    }
  }
}

void launch_resize_norm(const ResizeParams& p, hipStream_t s) {
  const size_t lds = (size_t)((3 * p.wi + 15) >> 4) * 16 * 2;
  hipLaunchKernelGGL(k_resize_norm, dim3(p.ho), dim3(256), lds, s, p);
}

// =============================================================================================
// Stage 2: implicit-GEMM convolution.  A workgroup (4 wavefronts) owns a 64-pixel x 64-channel
// output tile; each wavefront owns a 32x32 quarter and accumulates it with
// v_mfma_f32_32x32x16_f16.  The MFMA "A" operand is the weight tile and the "B" operand the
// pixel tile, so a lane ends up holding 4 consecutive output channels of one pixel per
// accumulator quad -> 8-byte fp16 stores into the pixel-major output.
// Global -> register prefetch of chunk q+1 overlaps the MFMAs of chunk q.
// =============================================================================================
template <int KC>
__global__ __launch_bounds__(256) void k_conv_mfma(ConvParams p) {
  constexpr int BM = 64, BN = 64;
  constexpr int PITCH = KC + 8;            // halves; +16 bytes keeps ds_read_b128 conflict-free
  constexpr int VPR = KC / 8;              // 16-byte vectors per tile row
  constexpr int NV = BM * VPR;             // vectors per tile (pixel tile and weight tile alike)
  constexpr int NP = (NV + 255) / 256;     // vectors per thread
  __shared__ __align__(16) f16 s_x[BM * PITCH];
  __shared__ __align__(16) f16 s_w[BN * PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int q_begin = blockIdx.z * p.chunks_per_split;
  const int q_end = min(p.nchunks, q_begin + p.chunks_per_split);

  // per-thread loader coordinates (fixed over the K loop)
  int l_row[NP], l_kv[NP], l_iy0[NP], l_ix0[NP];
  bool l_act[NP], l_ok[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int v = tid + i * 256;
    l_act[i] = v < NV;
    l_row[i] = v / VPR;
    l_kv[i] = v % VPR;
    const int m = m0 + l_row[i];
    l_ok[i] = l_act[i] && m < p.m;
    const int oy = m / p.wout, ox = m - oy * p.wout;
    l_iy0[i] = oy * p.stride - p.pad;
    l_ix0[i] = ox * p.stride - p.pad;
  }

  uint4 rx[NP], rw[NP];
  auto load_chunk = [&](int q) {
    const int tap = q / p.chunks_per_tap;
    const int cc = q - tap * p.chunks_per_tap;
    const int ky = tap / p.kw, kx = tap - ky * p.kw;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      if (!l_act[i]) continue;
      const int iy = l_iy0[i] + ky, ix = l_ix0[i] + kx;
      const bool inb = l_ok[i] && iy >= 0 && iy < p.hin && ix >= 0 && ix < p.win;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (inb) {
        const f16* a = p.in + ((size_t)iy * p.win + ix) * p.cin_pitch + cc * KC + l_kv[i] * 8;
        v = *reinterpret_cast<const uint4*>(a);
      }
      rx[i] = v;
      const f16* b = p.wt + (size_t)(n0 + l_row[i]) * p.ktot + (size_t)q * KC + l_kv[i] * 8;
      rw[i] = *reinterpret_cast<const uint4*>(b);
    }
  };

  floatx16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.0f;

  const int wm = wave & 1, wn = wave >> 1;
  const f16* fx = s_x + (wm * 32 + (lane & 31)) * PITCH + (lane >> 5) * 8;
  const f16* fw = s_w + (wn * 32 + (lane & 31)) * PITCH + (lane >> 5) * 8;

  if (q_begin < q_end) load_chunk(q_begin);
  for (int q = q_begin; q < q_end; ++q) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      if (!l_act[i]) continue;
      *reinterpret_cast<uint4*>(s_x + l_row[i] * PITCH + l_kv[i] * 8) = rx[i];
      *reinterpret_cast<uint4*>(s_w + l_row[i] * PITCH + l_kv[i] * 8) = rw[i];
    }
    __syncthreads();
    if (q + 1 < q_end) load_chunk(q + 1);
#pragma unroll
    for (int ks = 0; ks < KC / 16; ++ks) {
      const half8 a = *reinterpret_cast<const half8*>(fw + ks * 16);
      const half8 b = *reinterpret_cast<const half8*>(fx + ks * 16);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
    }
    __syncthreads();
  }

  // accumulator register 4*i + j holds channel n_base + 8*i + j of pixel m
  const int m = m0 + wm * 32 + (lane & 31);
  const int n_base = n0 + wn * 32 + (lane >> 5) * 4;
  if (m >= p.m) return;
  if (p.use_partial) {
    float* dst = p.partial + ((size_t)blockIdx.z * p.m + m) * p.cout_pad + n_base;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<float4*>(dst + 8 * i) =
          make_float4(acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]);
    return;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int n = n_base + 8 * i;
    if (n >= p.cout) continue;
    float v[4] = {acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]};
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
#pragma unroll
      for (int j = 0; j < 4; ++j) p.out_f32[(size_t)(n + j) * p.m + m] = v[j];
    } else {
      half4 o;
#pragma unroll
      for (int j = 0; j < 4; ++j) o[j] = (f16)v[j];
      *reinterpret_cast<half4*>(p.out + (size_t)m * p.out_pitch + n) = o;
    }
  }
}

void launch_conv_mfma(const ConvParams& p, hipStream_t s) {
  const dim3 grid((p.m + 63) / 64, p.cout_pad / 64, p.nsplit);
  if (p.kc == 16) hipLaunchKernelGGL(k_conv_mfma<16>, grid, dim3(256), 0, s, p);
  else if (p.kc == 32) hipLaunchKernelGGL(k_conv_mfma<32>, grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL(k_conv_mfma<64>, grid, dim3(256), 0, s, p);
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
#pragma unroll
    for (int j = 0; j < 4; ++j) p.out_f32[(size_t)(n + j) * p.m + m] = v[j];
  } else {
    half4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (f16)v[j];
    *reinterpret_cast<half4*>(p.out + (size_t)m * p.out_pitch + n) = o;
  }
}

void launch_splitk_epilogue(const SplitKEpilogueParams& p, hipStream_t s) {
  const size_t n = (size_t)p.m * (p.cout >> 2);
  hipLaunchKernelGGL(k_splitk_epilogue, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p);
}

// ---------------------------------------------------------------------------------------------
// ConvLSTM epilogue: one thread per (pixel, hidden channel); fp32 math, c kept in fp32.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float sigmoid_f(float x) { return 1.0f / (1.0f + __expf(-x)); }

__global__ __launch_bounds__(256) void k_lstm_epilogue(LstmEpilogueParams p) {
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)p.m * p.hid) return;
  const int m = (int)(t / p.hid), j = (int)(t - (size_t)m * p.hid);
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
  p.h_out[(size_t)m * p.h_pitch + j] = (f16)(go * tanhf(c_new));
}

void launch_lstm_epilogue(const LstmEpilogueParams& p, hipStream_t s) {
  const size_t n = (size_t)p.m * p.hid;
  hipLaunchKernelGGL(k_lstm_epilogue, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p);
}

// ---------------------------------------------------------------------------------------------
// Max-pool 3x3 / 2, pad 1: one thread per (output pixel, 8 channels).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_maxpool(MaxPoolParams p) {
  const int cv = p.c >> 3;
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)p.hout * p.wout * cv) return;
  const int v = (int)(t % cv);
  const int pix = (int)(t / cv);
  const int oy = pix / p.wout, ox = pix - oy * p.wout;
  half8 best;
  bool first = true;
  for (int ky = 0; ky < 3; ++ky) {
    const int iy = 2 * oy + ky - 1;
    if (iy < 0 || iy >= p.hin) continue;
    for (int kx = 0; kx < 3; ++kx) {
      const int ix = 2 * ox + kx - 1;
      if (ix < 0 || ix >= p.win) continue;
      const half8 x =
          *reinterpret_cast<const half8*>(p.in + ((size_t)iy * p.win + ix) * p.c + v * 8);
      if (first) { best = x; first = false; }
      else {
#pragma unroll
        for (int j = 0; j < 8; ++j) best[j] = x[j] > best[j] ? x[j] : best[j];
      }
    }
  }
  *reinterpret_cast<half8*>(p.out + (size_t)pix * p.c + v * 8) = best;
}

void launch_maxpool(const MaxPoolParams& p, hipStream_t s) {
  const size_t n = (size_t)p.hout * p.wout * (p.c >> 3);
  hipLaunchKernelGGL(k_maxpool, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p);
}

// ---------------------------------------------------------------------------------------------
// 1x1 head (8 output channels): one wavefront per pixel; lane l covers input channels
// l*8 .. l*8+7 (cin <= 512), butterfly-reduced with DPP-friendly shuffles.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_head(HeadParams p) {
  const int lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= p.m) return;
  float acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = 0.0f;
  for (int c0 = lane * 8; c0 < p.cin; c0 += 512) {
    const half8 x = *reinterpret_cast<const half8*>(p.h + (size_t)m * p.h_pitch + c0);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const half8 w = *reinterpret_cast<const half8*>(p.w + (size_t)k * p.cin + c0);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[k] += (float)x[j] * (float)w[j];
    }
  }
#pragma unroll
  for (int k = 0; k < 8; ++k) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc[k] += __shfl_xor(acc[k], off, 64);
  }
  if (lane < 8) {
    float v = acc[0];
#pragma unroll
    for (int k = 1; k < 8; ++k) v = (lane == k) ? acc[k] : v;
    p.logits[(size_t)lane * p.m + m] = v;
  }
}

void launch_head(const HeadParams& p, hipStream_t s) {
  hipLaunchKernelGGL(k_head, dim3((p.m + 3) / 4), dim3(256), 0, s, p);
}

// =============================================================================================
// Stage 3: one workgroup per tool channel.  Every lane keeps (best value, lowest index);
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
  const float* L = p.logits + (size_t)k * p.n;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = tid; i < p.n; i += 256) {
    const float x = L[i];
    p.heat[(size_t)k * p.n + i] = 1.0f / (1.0f + expf(-x));
    p.mask[(size_t)k * p.n + i] = x > p.theta ? 1 : 0;
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
    p.rec->argmax_idx[k] = bi;
    p.rec->peak[k] = 1.0f / (1.0f + expf(-bv));
    p.rec->present[k] = bv > p.theta ? 1 : 0;
  }
}

void launch_postprocess(const PostParams& p, hipStream_t s) {
  hipLaunchKernelGGL(k_postprocess, dim3(8), dim3(256), 0, s, p);
}

// =============================================================================================
// Stage 4: one workgroup per frame row.  The row's mask cells are reduced to "lowest set
// channel" once in LDS; each thread then streams 16 pixels (48 bytes) with 16-byte accesses.
// =============================================================================================
__global__ __launch_bounds__(128) void k_overlay(OverlayParams p) {
  extern __shared__ uint8_t s_k[];        // wm entries: lowest set channel or 0xff
  const int Y = blockIdx.x, tid = threadIdx.x;
  const int my = (int)(((long long)Y * p.hm) / p.hf);
  for (int x = tid; x < p.wm; x += 128) {
    uint8_t k = 0xff;
    for (int c = 7; c >= 0; --c)
      if (p.mask[((size_t)c * p.hm + my) * p.wm + x]) k = (uint8_t)c;
    s_k[x] = k;
  }
  __syncthreads();
  const uint8_t* srow = p.src + (size_t)Y * p.pitch;
  uint8_t* drow = p.dst + (size_t)Y * p.pitch;
  const int ia = 256 - p.a;
  for (int X0 = tid * 16; X0 < p.wf; X0 += 128 * 16) {
    const int npx = min(16, p.wf - X0);
    int mx = (int)(((long long)X0 * p.wm) / p.wf);
    int rem = (int)(((long long)X0 * p.wm) - (long long)mx * p.wf);
    if (npx == 16) {
      uint4 v[3];
      const uint4* s4 = reinterpret_cast<const uint4*>(srow + (size_t)X0 * 3);
      v[0] = s4[0]; v[1] = s4[1]; v[2] = s4[2];
      uint8_t* b = reinterpret_cast<uint8_t*>(v);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const uint8_t k = s_k[mx];
        if (k != 0xff) {
          const uint32_t col = p.pal[k];
#pragma unroll
          for (int c = 0; c < 3; ++c) {
            const uint32_t pc = (col >> (8 * c)) & 0xffu;
            b[3 * i + c] = (uint8_t)((p.a * pc + ia * (uint32_t)b[3 * i + c] + 128u) >> 8);
          }
        }
        rem += p.wm;
        while (rem >= p.wf) { rem -= p.wf; ++mx; }
      }
      uint4* d4 = reinterpret_cast<uint4*>(drow + (size_t)X0 * 3);
      d4[0] = v[0]; d4[1] = v[1]; d4[2] = v[2];
    } else {
      for (int i = 0; i < npx; ++i) {
        const uint8_t k = s_k[mx];
        for (int c = 0; c < 3; ++c) {
          uint32_t x = srow[(size_t)(X0 + i) * 3 + c];
          if (k != 0xff) {
            const uint32_t pc = (p.pal[k] >> (8 * c)) & 0xffu;
            x = (p.a * pc + ia * x + 128u) >> 8;
          }
          drow[(size_t)(X0 + i) * 3 + c] = (uint8_t)x;
        }
        rem += p.wm;
        while (rem >= p.wf) { rem -= p.wf; ++mx; }
      }
    }
  }
}

void launch_overlay(const OverlayParams& p, hipStream_t s) {
  hipLaunchKernelGGL(k_overlay, dim3(p.hf), dim3(128), (size_t)p.wm, s, p);
}

// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_fill_zero(uint4* d, size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride)
    d[i] = make_uint4(0, 0, 0, 0);
}

void launch_fill_zero(void* d, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 16;
  if (n == 0) return;
  const unsigned blocks = (unsigned)min((size_t)2048, (n + 255) / 256);
  hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, s, reinterpret_cast<uint4*>(d), n);
}

}  // namespace hs
