// libhs host runtime: contexts, applications, the per-frame launch plan, CU-masked stream
// partitions with admission control, per-frame time stamps and the completion thread.
// Paper: Section III-A (application and its four stages), Section II-C (time stamps at the
// first and last stage), Section IV-A (exclusive partitions, admission control).
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <condition_variable>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <stdexcept>
#include <string>
#include <thread>
#include <pthread.h>
#include <sched.h>
#include <time.h>
#include <unistd.h>
#include <vector>

#include "hs.h"
#include "hs_internal.h"
#include "hs_kernels.h"

namespace hs {

static inline uint64_t now_ns() {
  timespec ts;
  clock_gettime(CLOCK_MONOTONIC, &ts);
  return (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
}

#define HS_HIP(call)                                                                   \
  do {                                                                                 \
    hipError_t e_ = (call);                                                            \
    if (e_ != hipSuccess) {                                                            \
      set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
      return HS_E_DEVICE;                                                              \
    }                                                                                  \
  } while (0)

// ---- kernel families (for timing) ----------------------------------------------------------
enum Family { F_RESIZE, F_CONV, F_SPLITK, F_LSTM, F_STEM, F_POST, F_OVERLAY, F_COUNT };
static const char* kFamilyName[F_COUNT] = {"resize_norm", "conv_mfma", "splitk_epilogue",
                                           "lstm_head", "stem_pool_mfma", "postprocess", "overlay"};

struct Op {
  Family fam;
  double flops = 0, bytes = 0;
  ResizeParams resize;
  ConvParams conv;
  SplitKEpilogueParams splitk;
  LstmEpilogueParams lstm;
  StemPoolParams stem;
  PostParams post;
  OverlayParams overlay;
};

static KernelDesc op_desc(const Op& op) {
  switch (op.fam) {
    case F_RESIZE: return describe(op.resize);
    case F_CONV: return describe(op.conv);
    case F_SPLITK: return describe(op.splitk);
    case F_LSTM: return describe(op.lstm);
    case F_STEM: return describe(op.stem);
    case F_POST: return describe(op.post);
    default: return describe(op.overlay);
  }
}

static void* op_params(Op& op) {
  switch (op.fam) {
    case F_RESIZE: return &op.resize;
    case F_CONV: return &op.conv;
    case F_SPLITK: return &op.splitk;
    case F_LSTM: return &op.lstm;
    case F_STEM: return &op.stem;
    case F_POST: return &op.post;
    default: return &op.overlay;
  }
}

static hipError_t launch_op(Op& op, hipStream_t s) {
  const KernelDesc d = op_desc(op);
  void* args[1] = {op_params(op)};
  return hipLaunchKernel(d.func, d.grid, d.block, args, d.shmem, s);
}

// ---- workspace carving -----------------------------------------------------------------------
struct Carver {
  uint8_t* base;   // may be NULL for a dry run
  size_t off = 0;
  explicit Carver(void* b) : base((uint8_t*)b) {}
  template <typename T>
  T* take(size_t count) {
    off = (off + 255) & ~(size_t)255;
    T* p = base ? (T*)(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

struct Tensor {
  f16* p = nullptr;
  int h = 0, w = 0, c = 0, pitch = 0;
};

enum SlotState { SLOT_FREE = 0, SLOT_INFLIGHT = 1, SLOT_DONE = 2 };
// Two lanes: with more frames in flight the submitting host thread (one graph launch per frame,
// about 75 us) is the limit, not the GPU (four lanes were measured: no gain).
constexpr int kMaxLanes = 2;

struct Slot {
  std::vector<Op> pre;     // stage 1: one launch, blockIdx.y = stream of the batch
  std::vector<Op> infer;   // stage 2: the network over the whole batch
  std::vector<Op> infer_static;   // the same with the split-K scratch in the library's fixed
                                  // device array (empty when the scratch needed exceeds it)
  std::vector<Op> post;    // stage 3
  std::vector<Op> overlay; // stage 4: one launch, blockIdx.y = stream of the batch
  hipEvent_t ev_pre = nullptr, ev_infer = nullptr, ev_post = nullptr, ev_overlay = nullptr;
  // Consecutive frames rotate over the lanes (activation sets + streams) and overlap;
  // the recurrent cell is the only thing that chains them: its gate convolution (op wait_idx)
  // waits for the previous frame's state update, whose kernel (op record_idx) is followed by a
  // record of ev_state.  -1: the network has no recurrent state.
  int lane = 0, wait_idx = -1, record_idx = -1;
  hipEvent_t ev_state = nullptr;
  // stages 1-3 as one HIP graph (kernel nodes chained in order, event-record nodes at the
  // stage boundaries); only the frame pointer of the first node changes from frame to frame
  hipGraph_t graph = nullptr;
  hipGraphExec_t graph_exec = nullptr;
  std::vector<hipGraphNode_t> resize_nodes;
  PostRecord* rec = nullptr;   // [batch], pinned host memory, written by the stage-3 kernel
  f16* d_netin = nullptr;      // [batch] padded images
  float* d_netin_f32 = nullptr;
  float* d_logits = nullptr;   // [batch][8][n]
  float* d_heat = nullptr;
  uint8_t* d_mask = nullptr;
  int state = SLOT_FREE;
  std::vector<hs_result> results;   // one per stream of the batch
};

struct TimedLaunch {
  Family fam;
  double flops, bytes;
  hipEvent_t e0, e1;
};

}  // namespace hs

using namespace hs;

struct hs_ctx {
  int device = 0;
  int n_cus = 0;
  void* d_static_scratch = nullptr;   // the library's fixed scratch array on this device
  size_t static_scratch_bytes = 0;
  std::mutex mu;
  std::vector<hs_app*> apps;
};

struct hs_app {
  hs_ctx* ctx = nullptr;
  hs_app_desc desc;
  int map_w = 0, map_h = 0;
  int batch = 1;
  int netin_w = 0, netin_h = 0, netin_pad = 0;   // padded stage-1 output geometry
  bool stateful = false;
  // recurrent state
  float* d_c = nullptr;
  f16* d_concat[kMaxLanes] = {nullptr};   // per lane: [x_t ; h_{t-1}] of the frames that run there
  int concat_pitch = 0, hid = 0, x_ch = 0;
  int lanes = 1;
  hipStream_t lane_last_stream[kMaxLanes] = {nullptr};   // stream each lane's latest frame used
  // streams / partition: s_lane[i] carries lane i (all equal to s_lane[0] when partitioned, so
  // that a partition keeps to one hardware queue); s_overlay is NULL when the overlay follows
  // its frame's lane stream
  hipStream_t s_lane[kMaxLanes] = {nullptr};
  hipStream_t s_overlay = nullptr;
  bool partitioned = false;
  uint32_t claim[HS_MAX_CU_WORDS] = {0};
  // ring
  std::vector<Slot> slots;
  int depth = 0;
  uint64_t n_submitted = 0, n_completed = 0, n_delivered = 0;
  std::mutex mu;
  std::condition_variable cv_work, cv_done;
  std::thread completer;
  bool stop = false;
  std::string completer_error;
  int launch_mode = HS_LAUNCH_EAGER;
  // kernel timing
  bool timing = false;
  std::vector<TimedLaunch> timed;
  double acc_ms[F_COUNT] = {0}, acc_flops[F_COUNT] = {0}, acc_bytes[F_COUNT] = {0};
  uint64_t acc_n[F_COUNT] = {0};
  void* pinned = nullptr;
  hs_group* group = nullptr;   // set while the application is a member of a multi-network group
  size_t partial_bytes = 0;    // split-K scratch one frame needs
};

// A multi-network application: the members run stages 1-3 on the same frame side by side, one
// overlay launch of the group draws all their layers.
// The paper's inference operator launches the parallel inferences from one CPU thread each
// (Section III-B); likewise every member but the first has a thread that enqueues its stages
// 1-3 while the caller's thread enqueues the first member's, so the host launch costs overlap.
struct GroupWorker {
  std::thread th;
  std::mutex mu;
  std::condition_variable cv;
  bool has_job = false, done = false, stop = false;
  // the job: one frame for member `app`
  hs_app* app = nullptr;
  const uint8_t* d_frame = nullptr;
  uint8_t* d_out = nullptr;
  uint64_t frame_id = 0, t_submit = 0;
  // its outcome
  hs_status status = HS_OK;
  std::string error;
  Slot* slot = nullptr;
  hipStream_t tail = nullptr;
};

struct hs_group {
  hs_ctx* ctx = nullptr;
  std::vector<hs_app*> members;
  std::vector<Op> overlay;   // one op; its layers are refilled from the members' slots per frame
  std::vector<std::unique_ptr<GroupWorker>> workers;   // workers[i] serves members[i + 1]
};

namespace hs {

// ---- weight packing ----------------------------------------------------------------------------
// Generic layer: packed[n][(ky*k + kx)*cin + c] = w[n][c][ky][kx]; rows cout..cout_pad-1 zero.
static void pack_generic(const float* w, int cout, int cin, int k, int cout_pad, f16* dst) {
  const size_t ktot = (size_t)k * k * cin;
  std::memset(dst, 0, (size_t)cout_pad * ktot * sizeof(f16));
  for (int n = 0; n < cout; ++n)
    for (int c = 0; c < cin; ++c)
      for (int ky = 0; ky < k; ++ky)
        for (int kx = 0; kx < k; ++kx)
          dst[(size_t)n * ktot + (size_t)(ky * k + kx) * cin + c] =
              (f16)w[(((size_t)n * cin + c) * k + ky) * k + kx];
}

// The same layer in MFMA fragment order for the kernel that reads its weight operand straight
// from memory (3x3, cin % 64 == 0): dst[(((g*chunks + cc)*9 + tap)*4 + ks)*64 + lane][j] =
// w[32*g + r][64*cc + 16*ks + 8*h + j][tap], lane = r + 32*h; channels above cout are zero.
// ntaps = 9 (3x3) or 1 (the 1x1 projection fused into a stride-2 layer).
static void pack_frag(const float* w, int cout, int cin, int ntaps, int cout_pad, f16* dst) {
  const int chunks = cin / 64;
  std::memset(dst, 0, (size_t)cout_pad * ntaps * cin * sizeof(f16));
  for (int n = 0; n < cout; ++n) {
    const int g = n / 32, r = n % 32;
    for (int c = 0; c < cin; ++c) {
      const int cc = c / 64, ks = (c % 64) / 16, h = (c % 16) / 8, j = c % 8;
      for (int tap = 0; tap < ntaps; ++tap) {
        const size_t block = (((size_t)g * chunks + cc) * ntaps + tap) * 4 + ks;
        dst[(block * 64 + (size_t)(r + 32 * h)) * 8 + j] =
            (f16)w[((size_t)n * cin + c) * ntaps + tap];
      }
    }
  }
}

// First layer on the padded 4-channel image: one chunk per kernel row, covering chunk_px
// adjacent pixels of 4 channels; packed[n][ky][px][ch] = w[n][ch][ky][px] (px < k, ch < 3).
static void pack_rowtap(const float* w, int cout, int k, int chunk_px, int cout_pad, f16* dst) {
  const size_t ktot = (size_t)k * chunk_px * 4;
  std::memset(dst, 0, (size_t)cout_pad * ktot * sizeof(f16));
  for (int n = 0; n < cout; ++n)
    for (int ch = 0; ch < 3; ++ch)
      for (int ky = 0; ky < k; ++ky)
        for (int px = 0; px < k; ++px)
          dst[(size_t)n * ktot + ((size_t)ky * chunk_px + px) * 4 + ch] =
              (f16)w[(((size_t)n * 3 + ch) * k + ky) * k + px];
}

// The 7x7 stem's weights in MFMA fragment order for k_stem_pool: block ((wn * 7 + ky) * 2 + s) of
// 64 lanes x 8 halves; lane (h, r) holds channel 32 * wn + r, k = ky * 32 + s * 16 + h * 8 .. + 7 of
// the row-tap layout (k = (ky * 8 + px) * 4 + ch, zero where px == 7 or ch == 3).
static void pack_stem_frag(const float* w, f16* dst) {
  std::vector<f16> rows((size_t)64 * 224);
  pack_rowtap(w, 64, 7, 8, 64, rows.data());
  for (int wn = 0; wn < 2; ++wn)
    for (int ky = 0; ky < 7; ++ky)
      for (int s = 0; s < 2; ++s)
        for (int lane = 0; lane < 64; ++lane) {
          const int h = lane >> 5, r = lane & 31;
          const f16* src = rows.data() + (size_t)(32 * wn + r) * 224 + ky * 32 + s * 16 + h * 8;
          f16* out = dst + ((size_t)((wn * 7 + ky) * 2 + s) * 64 + lane) * 8;
          for (int e = 0; e < 8; ++e) out[e] = src[e];
        }
}

// ---- plan builder ------------------------------------------------------------------------------
static inline int conv_out(int n, int k, int s, int p) { return (n + 2 * p - k) / s + 1; }
static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
static inline size_t round_up_sz(size_t v, size_t m) { return (v + m - 1) / m * m; }

// Walks the layers of a network in blob order.  Used twice: a sizing walk (no pointers, no
// packing) that yields the packed-weight and split-K scratch sizes, then the real walk.
struct Builder {
  const hs_app_desc& d;
  Carver carve;
  bool pack;                      // pack weights on the host (create only)
  bool carve_acts;                // hand out activation storage (second walk)
  std::vector<f16> host_w;        // packed weights staged on the host
  f16* d_w = nullptr;             // device weights base
  size_t w_halves = 0;            // packed weights consumed so far
  const float* blob;
  size_t blob_off = 0;
  size_t partial_floats = 0;
  float* d_partial = nullptr;     // split-K scratch of this lane inside the workspace
  std::vector<Op> ops;            // stage-2 ops; slot-dependent pointers are patched per slot
  int first_conv_op = -1;         // op whose conv.in is the slot's padded net input
  int logits_op = -1;             // op that writes the slot's logits
  int lstm_conv_op = -1;          // gate convolution of the recurrent cell (-1: none)
  int map_h = 0, map_w = 0;
  bool stateful = false;
  float* d_c = nullptr;
  f16* d_concat = nullptr;

  Builder(const hs_app_desc& desc, void* base, bool do_pack, bool do_carve)
      : d(desc), carve(base), pack(do_pack), carve_acts(do_carve), blob(desc.weights) {}

  template <typename T>
  T* acts(size_t count) { return carve_acts ? carve.take<T>(count) : nullptr; }

  // Reserve room for n packed halves; returns the offset. Regions start 256-byte aligned.
  size_t reserve_w(size_t n) {
    const size_t off = w_halves;
    w_halves = round_up_sz(off + n, 128);
    if (pack) host_w.resize(w_halves);
    return off;
  }

  // Picks the kernel variant, the tile grid and the split along K.
  static void choose_split(ConvParams& c) {
    // the shared-patch kernels address the input with 32-bit offsets (in halves)
    const bool fits32 = (double)c.batch * c.hin * c.win * c.cin_pitch < 2147483648.0;
    const bool halo = c.ntaps == 9 && c.kw == 3 && c.stride == 1 && c.pad == 1 && c.kc == 64 && fits32;
    const bool halo2 = c.ntaps == 9 && c.kw == 3 && c.stride == 2 && c.pad == 1 && c.kc == 64 && fits32;
    if (halo2) {
      c.variant = 4;
      c.tiles_x = (c.wout + 7) / 8;
      c.tiles_m = c.batch * ((c.hout + 7) / 8) * c.tiles_x;
      c.tiles_n = c.cout_pad / 64;
      const int tiles = c.tiles_m * c.tiles_n;
      // from 1.5 workgroups per CU on: weights as fragments from memory, half-chunk patches
      // (channel tiles of 128 there: the patch, the heavy operand at stride 2, serves them all)
      if (tiles >= 768 && c.frag_ok && c.cout % 128 == 0) {
        c.variant = 7;
        c.tiles_n = c.cout_pad / 128;
      }
      const int units = c.chunks_per_tap;
      int ns = 1;
      if (tiles < 192) ns = std::max(1, std::min((256 + tiles - 1) / tiles, units));
      c.chunks_per_split = (units + ns - 1) / ns;
      c.nsplit = (units + c.chunks_per_split - 1) / c.chunks_per_split;
    } else if (halo) {
      // spatial tiles of 8 x 16 pixels when that still yields enough workgroups, else 8 x 8;
      // grids of more than two workgroups per CU take the leaner 8 x 16 kernel (three per CU)
      const int ty = (c.hout + 7) / 8;
      const int wide = c.batch * ty * ((c.wout + 15) / 16) * (c.cout_pad / 64);
      c.variant = wide > 512 ? 3 : wide >= 192 ? 2 : 1;
      // from 1.5 workgroups per CU on, layers with several Cin chunks are paced by LDS
      // throughput: the variant that keeps the weights out of LDS takes them
      if (wide >= 384 && c.chunks_per_tap >= 2) c.variant = 6;
      const int tw = c.variant == 1 ? 8 : 16;
      c.tiles_x = (c.wout + tw - 1) / tw;
      c.tiles_m = c.batch * ty * c.tiles_x;
      c.tiles_n = c.cout_pad / 64;
      const int tiles = c.tiles_m * c.tiles_n;
      const int units = c.chunks_per_tap;        // split over Cin chunks
      int ns = 1;
      if (tiles < 192) ns = std::max(1, std::min((256 + tiles - 1) / tiles, units / 2));
      c.chunks_per_split = (units + ns - 1) / ns;
      c.nsplit = (units + c.chunks_per_split - 1) / c.chunks_per_split;
    } else {
      c.variant = 0;
      c.tiles_x = 0;
      c.tiles_m = (c.m + 63) / 64;
      c.tiles_n = c.cout_pad / 64;
      const int tiles = c.tiles_m * c.tiles_n;
      int ns = 1;
      if (tiles < 192) ns = std::max(1, std::min((320 + tiles - 1) / tiles, c.nchunks / 4));
      c.chunks_per_split = (c.nchunks + ns - 1) / ns;
      c.nsplit = (c.nchunks + c.chunks_per_split - 1) / c.chunks_per_split;
    }
    c.depth = (c.kc == 64 && c.chunks_per_split >= 12) ? 8 : 4;
    // grids several times what the device holds at once (768 workgroups): each workgroup walks
    // consecutive spatial tiles, sized so that the whole grid is resident at two per CU
    c.tiles_per_wg = 1;
    if (c.variant == 3 || c.variant == 4) {
      const int wgs = c.tiles_m * c.tiles_n * c.nsplit;
      if (wgs > 1536) c.tiles_per_wg = (wgs + 511) / 512;
    }
    if (c.variant == 7) {   // two workgroups per CU are resident: beyond two rounds, walk in one
      const int wgs = c.tiles_m * c.tiles_n * c.nsplit;
      if (wgs > 1024) c.tiles_per_wg = (wgs + 511) / 512;
    }
    const int groups_m = (c.tiles_m + c.tiles_per_wg - 1) / c.tiles_per_wg;
    c.tiles_per_xcd = (groups_m * c.tiles_n * c.nsplit + 7) / 8;
    // Tile order: every XCD (own L2) takes a run of tiles_per_xcd consecutive tiles.  For every
    // block size, count what the eight L2s fetch (each its own spatial groups' input slices and
    // its own channel tiles' weight slices, once) and keep the cheapest.
    c.n_block = 1;
    if (((c.variant >= 1 && c.variant <= 4) || c.variant == 6 || c.variant == 7) && c.tiles_n > 1) {
      const double in_unit = 2.0 * c.batch * c.hin * c.win * (c.chunks_per_tap * 64.0) /
                             ((double)groups_m * c.nsplit);
      const double w_unit = 2.0 * c.cout_pad * c.ktot / ((double)c.tiles_n * c.nsplit);
      const int per_split = groups_m * c.tiles_n, total = per_split * c.nsplit;
      double best = 0;
      for (int nb = 1; nb <= c.tiles_n; nb *= 2) {
        if (c.tiles_n % nb) continue;
        double bytes = 0;
        std::vector<char> seen_in((size_t)groups_m * c.nsplit), seen_w((size_t)c.tiles_n * c.nsplit);
        for (int x = 0; x < 8; ++x) {
          std::fill(seen_in.begin(), seen_in.end(), 0);
          std::fill(seen_w.begin(), seen_w.end(), 0);
          for (int t = x * c.tiles_per_xcd; t < std::min(total, (x + 1) * c.tiles_per_xcd); ++t) {
            const int split = t / per_split, within = t % per_split;
            const int blk = groups_m * nb, in_blk = within % blk;
            const int gm = in_blk / nb, tn = (within / blk) * nb + in_blk % nb;
            char& si = seen_in[(size_t)split * groups_m + gm];
            char& sw = seen_w[(size_t)split * c.tiles_n + tn];
            if (!si) { si = 1; bytes += in_unit; }
            if (!sw) { sw = 1; bytes += w_unit; }
          }
        }
        if (nb == 1 || bytes < 0.9 * best) { best = bytes; c.n_block = nb; }
      }
    }
  }

  // Appends the convolution and, when it is split along K, its reduction kernel.
  // keep_partial: leave the partial sums in the scratch buffer for a later kernel (ConvLSTM).
  // Returns the index of the convolution op.
  // w2_off / out2: packed weights and output of a 1x1 stride-2 projection fused into a 3x3
  // stride-2 layer (out2 == NULL: none).
  int add_conv(ConvParams c, size_t w_off, const Tensor* res, const Tensor* out, bool relu,
               bool want_f32, bool keep_partial, double flops, size_t w2_off = 0,
               const Tensor* out2 = nullptr, size_t wf_off = (size_t)-1,
               size_t wf2_off = (size_t)-1) {
    Op op;
    op.fam = F_CONV;
    op.flops = flops;
    c.wt = d_w ? d_w + w_off : nullptr;
    c.wt_frag = (d_w && wf_off != (size_t)-1) ? d_w + wf_off : nullptr;
    choose_split(c);
    const bool partial = c.nsplit > 1 || keep_partial;
    c.use_partial = partial ? 1 : 0;
    c.partial = nullptr;   // patched when the scratch buffer is carved
    c.out = nullptr; c.out_pitch = 0; c.res = nullptr; c.res_pitch = 0; c.relu = 0;
    c.out_f32 = nullptr;
    c.wt2 = nullptr; c.out2 = nullptr; c.out2_pitch = 0; c.partial2 = nullptr;
    const bool fused = out2 != nullptr && (c.variant == 4 || c.variant == 7);
    c.wt2_frag = nullptr;
    if (fused) {
      c.wt2 = d_w ? d_w + w2_off : nullptr;
      c.wt2_frag = (d_w && wf2_off != (size_t)-1) ? d_w + wf2_off : nullptr;
      if (!partial) { c.out2 = out2->p; c.out2_pitch = out2->pitch; }
    }
    if (partial) {
      partial_floats =
          std::max(partial_floats, (size_t)(fused ? 2 : 1) * c.nsplit * c.m * c.cout_pad);
    } else {
      if (out) { c.out = out->p; c.out_pitch = out->pitch; }
      if (res) { c.res = res->p; c.res_pitch = res->pitch; }
      c.relu = relu ? 1 : 0;
    }
    op.conv = c;
    ops.push_back(op);
    const int conv_idx = (int)ops.size() - 1;
    if (want_f32 && !partial) logits_op = conv_idx;
    if (partial && !keep_partial) {
      Op e;
      e.fam = F_SPLITK;
      e.bytes = (double)c.nsplit * c.m * c.cout * 4.0 + (double)c.m * c.cout * 2.0;
      SplitKEpilogueParams& s = e.splitk;
      s.partial = nullptr;
      s.nsplit = c.nsplit; s.m = c.m; s.cout = c.cout; s.cout_pad = c.cout_pad;
      s.out = out ? out->p : nullptr; s.out_pitch = out ? out->pitch : 0;
      s.res = res ? res->p : nullptr; s.res_pitch = res ? res->pitch : 0;
      s.relu = relu ? 1 : 0;
      s.out_f32 = nullptr;
      s.img_m = c.img_m;
      s.partial2 = nullptr; s.out2 = nullptr; s.out2_pitch = 0;
      if (fused) {
        s.out2 = out2->p; s.out2_pitch = out2->pitch;   // partial2 patched with the scratch
        e.bytes *= 2.0;
      }
      ops.push_back(e);
      if (want_f32) logits_op = (int)ops.size() - 1;
    }
    return conv_idx;
  }

  // Generic convolution on a pixel-major tensor; weights are the next cout*cin*k*k floats of the
  // blob starting at blob_at. Fills out->h/w/c.
  // proj_at / proj_out: blob offset and output of the block's 1x1 stride-2 projection, fused into
  // this 3x3 stride-2 layer when the layer qualifies (returns through *proj_fused whether it was).
  int conv_layer(const Tensor& in, size_t blob_at, int cout, int k, int stride, int pad, bool relu,
                 const Tensor* res, Tensor* out, bool want_f32, bool keep_partial,
                 size_t proj_at = 0, Tensor* proj_out = nullptr, bool* proj_fused = nullptr) {
    const int cin = in.c;
    ConvParams g;
    std::memset(&g, 0, sizeof(g));
    g.in = in.p; g.hin = in.h; g.win = in.w; g.cin_pitch = in.pitch;
    g.hout = conv_out(in.h, k, stride, pad); g.wout = conv_out(in.w, k, stride, pad);
    g.batch = d.batch; g.img_m = g.hout * g.wout; g.m = g.batch * g.img_m;
    g.cout = cout; g.cout_pad = round_up(cout, 64);
    g.kc = (cin % 64 == 0) ? 64 : (cin % 32 == 0 ? 32 : 16);
    g.ntaps = k * k; g.kw = k; g.chunks_per_tap = cin / g.kc;
    g.nchunks = g.ntaps * g.chunks_per_tap; g.ktot = g.nchunks * g.kc;
    g.stride = stride; g.pad = pad;
    g.frag_ok = (res == nullptr && !want_f32) ? 1 : 0;
    const size_t w_off = reserve_w((size_t)g.cout_pad * g.ktot);
    if (pack) pack_generic(blob + blob_at, cout, cin, k, g.cout_pad, host_w.data() + w_off);
    out->h = g.hout; out->w = g.wout; out->c = cout;
    const bool fuse = proj_out && k == 3 && stride == 2 && pad == 1 && g.kc == 64 &&
                      (double)g.batch * g.hin * g.win * g.cin_pitch < 2147483648.0;
    if (proj_fused) *proj_fused = fuse;
    if (!fuse) {
      // the kernel variant is a function of the shapes alone: layers that will read their
      // weights as MFMA fragments get a second, fragment-ordered copy
      size_t wf_off = (size_t)-1;
      ConvParams probe = g;
      choose_split(probe);
      if (probe.variant == 6 || probe.variant == 7) {
        wf_off = reserve_w((size_t)g.cout_pad * g.ktot);
        if (pack) pack_frag(blob + blob_at, cout, cin, 9, g.cout_pad, host_w.data() + wf_off);
      }
      return add_conv(g, w_off, res, out, relu, want_f32, keep_partial,
                      2.0 * g.m * (double)cout * cin * k * k, 0, nullptr, wf_off);
    }
    const size_t w2_off = reserve_w((size_t)g.cout_pad * cin);
    if (pack) pack_generic(blob + proj_at, cout, cin, 1, g.cout_pad, host_w.data() + w2_off);
    proj_out->h = g.hout; proj_out->w = g.wout; proj_out->c = cout;
    size_t wf_off = (size_t)-1, wf2_off = (size_t)-1;
    ConvParams probe = g;
    choose_split(probe);
    if (probe.variant == 7) {   // fragment-ordered copies of the 3x3 weights and of the projection
      wf_off = reserve_w((size_t)g.cout_pad * g.ktot);
      wf2_off = reserve_w((size_t)g.cout_pad * cin);
      if (pack) {
        pack_frag(blob + blob_at, cout, cin, 9, g.cout_pad, host_w.data() + wf_off);
        pack_frag(blob + proj_at, cout, cin, 1, g.cout_pad, host_w.data() + wf2_off);
      }
    }
    return add_conv(g, w_off, res, out, relu, want_f32, keep_partial,
                    2.0 * g.m * (double)cout * cin * (k * k + 1), w2_off, proj_out, wf_off, wf2_off);
  }

  // A 64 -> 64 -> 64 channel BasicBlock without projection as ONE launch (k_block64_fused):
  // out = ReLU(conv_b(ReLU(conv_a(in))) + in).  For grids up to the size from which the layers
  // walk their tiles (measured: 3-9 % more frames per second at 1 to 6 frames per launch, even
  // from 8 on, where the tile-walking kernel with resident weights takes over).
  // Weights are reserved in blob order (conv a, conv b), as by two conv_layer calls.
  static bool block64_fits(const hs_app_desc& d, const Tensor& in) {
    const long tiles = (long)d.batch * ((in.h + 7) / 8) * ((in.w + 15) / 16);
    return in.c == 64 && tiles <= 1536 &&
           (double)d.batch * in.h * in.w * in.pitch < 2147483648.0;
  }
  void block64_layer(const Tensor& in, size_t at_a, size_t at_b, Tensor* out) {
    ConvParams g;
    std::memset(&g, 0, sizeof(g));
    g.in = in.p; g.hin = in.h; g.win = in.w; g.cin_pitch = in.pitch;
    g.hout = in.h; g.wout = in.w;
    g.batch = d.batch; g.img_m = g.hout * g.wout; g.m = g.batch * g.img_m;
    g.cout = 64; g.cout_pad = 64; g.kc = 64;
    g.ntaps = 9; g.kw = 3; g.chunks_per_tap = 1; g.nchunks = 9; g.ktot = 576;
    g.stride = 1; g.pad = 1;
    const size_t wa_off = reserve_w((size_t)64 * 576);
    if (pack) pack_generic(blob + at_a, 64, 64, 3, 64, host_w.data() + wa_off);
    const size_t wb_off = reserve_w((size_t)64 * 576);
    if (pack) pack_generic(blob + at_b, 64, 64, 3, 64, host_w.data() + wb_off);
    out->h = g.hout; out->w = g.wout; out->c = 64;
    g.variant = 5;
    g.tiles_x = (g.wout + 15) / 16;
    g.tiles_m = g.batch * ((g.hout + 7) / 8) * g.tiles_x;
    g.tiles_n = 1; g.nsplit = 1; g.chunks_per_split = 1; g.tiles_per_wg = 1; g.n_block = 1;
    g.depth = 4;
    g.tiles_per_xcd = (g.tiles_m + 7) / 8;
    g.wt = d_w ? d_w + wa_off : nullptr;
    g.wt2 = d_w ? d_w + wb_off : nullptr;
    g.out = out->p; g.out_pitch = out->pitch;
    g.res = in.p; g.res_pitch = in.pitch;
    g.relu = 1;
    Op op;
    op.fam = F_CONV;
    op.flops = 2.0 * (2.0 * g.m * 64.0 * 64.0 * 9.0);
    op.conv = g;
    ops.push_back(op);
  }

  // First layer: 3 input channels on the padded 4-channel image, k x k, stride 2, ReLU.
  void first_layer(size_t blob_at, int pad_img_h, int pad_img_w, int cout, int k, Tensor* out) {
    const int pad = k / 2;
    const int chunk_px = (k <= 4) ? 4 : 8;
    ConvParams g;
    std::memset(&g, 0, sizeof(g));
    g.in = nullptr;   // per slot
    g.hin = pad_img_h; g.win = pad_img_w; g.cin_pitch = 4;
    g.hout = conv_out(d.net_h, k, 2, pad); g.wout = conv_out(d.net_w, k, 2, pad);
    g.batch = d.batch; g.img_m = g.hout * g.wout; g.m = g.batch * g.img_m;
    g.cout = cout; g.cout_pad = round_up(cout, 64);
    g.kc = chunk_px * 4;
    g.ntaps = k; g.kw = 1; g.chunks_per_tap = 1; g.nchunks = k; g.ktot = k * g.kc;
    g.stride = 2; g.pad = 0;
    const size_t w_off = reserve_w((size_t)g.cout_pad * g.ktot);
    if (pack) pack_rowtap(blob + blob_at, cout, k, chunk_px, g.cout_pad, host_w.data() + w_off);
    out->h = g.hout; out->w = g.wout; out->c = cout;
    first_conv_op =
        add_conv(g, w_off, nullptr, out, true, false, false, 2.0 * g.m * (double)cout * 3 * k * k);
  }

  void walk_tiny(int ph, int pw) {
    const int h1 = conv_out(d.net_h, 3, 2, 1), w1 = conv_out(d.net_w, 3, 2, 1);
    const int h2 = conv_out(h1, 3, 2, 1), w2 = conv_out(w1, 3, 2, 1);
    Tensor t1, t2, t3, lg;
    const size_t nb = (size_t)d.batch;
    t1.p = acts<f16>(nb * h1 * w1 * 16); t1.pitch = 16;
    t2.p = acts<f16>(nb * h2 * w2 * 32); t2.pitch = 32;
    t3.p = acts<f16>(nb * h2 * w2 * 32); t3.pitch = 32;
    size_t at = 0;
    first_layer(at, ph, pw, 16, 3, &t1);                                 at += 16 * 3 * 9;
    conv_layer(t1, at, 32, 3, 2, 1, true, nullptr, &t2, false, false);   at += 32 * 16 * 9;
    conv_layer(t2, at, 32, 3, 1, 1, true, nullptr, &t3, false, false);   at += 32 * 32 * 9;
    conv_layer(t3, at, 8, 3, 1, 1, false, nullptr, &lg, true, false);    at += 8 * 32 * 9;
    blob_off = at;
    map_h = lg.h; map_w = lg.w; stateful = false;
  }

  void walk_resnet(int ph, int pw) {
    const int hs_ = conv_out(d.net_h, 7, 2, 3), ws_ = conv_out(d.net_w, 7, 2, 3);
    const int hp = conv_out(hs_, 3, 2, 1), wp = conv_out(ws_, 3, 2, 1);
    int hf = hp, wf = wp;
    for (int i = 0; i < 3; ++i) { hf = conv_out(hf, 3, 2, 1); wf = conv_out(wf, 3, 2, 1); }
    const size_t nb = (size_t)d.batch;
    const int mf = (int)nb * hf * wf;                    // feature-map pixels over the batch
    Tensor buf[4];
    for (int i = 0; i < 4; ++i) buf[i].p = acts<f16>(nb * hp * wp * 64);
    f16* concat = acts<f16>((size_t)mf * 768);
    float* cstate = acts<float>((size_t)mf * 256);

    size_t at = 0;
    {
      // stem convolution and max-pool in one kernel; weights packed as MFMA fragments of row
      // taps of 8 pixels
      const size_t w_off = reserve_w((size_t)64 * 224);
      if (pack) pack_stem_frag(blob + at, host_w.data() + w_off);
      Op op;
      op.fam = F_STEM;
      StemPoolParams& sp = op.stem;
      std::memset(&sp, 0, sizeof(sp));
      sp.in = nullptr;   // per slot
      sp.wt = d_w ? d_w + w_off : nullptr;
      sp.out = buf[0].p;
      sp.hin = ph; sp.win = pw; sp.hc = hs_; sp.wc = ws_; sp.hp = hp; sp.wp = wp;
      sp.batch = d.batch;
      sp.tiles_x = (wp + 14) / 15; sp.tiles_y = (hp + 7) / 8;
      sp.tiles_per_xcd = (sp.batch * sp.tiles_x * sp.tiles_y + 7) / 8;
      op.flops = 2.0 * nb * hs_ * ws_ * 64.0 * 3 * 49;
      op.bytes = nb * ((double)d.net_h * d.net_w * 8 + (double)hp * wp * 64 * 2);
      ops.push_back(op);
      first_conv_op = (int)ops.size() - 1;
    }
    at += 64 * 3 * 49;
    int cur = 0;
    buf[0].h = hp; buf[0].w = wp; buf[0].c = 64; buf[0].pitch = 64;
    const int widths[4] = {64, 128, 256, 512};
    int cin = 64;
    for (int s = 0; s < 4; ++s) {
      for (int blk = 0; blk < 2; ++blk) {
        const int width = widths[s];
        const bool proj = blk == 0 && cin != width;
        const int bc_in = blk == 0 ? cin : width;
        const Tensor a = buf[cur];
        Tensor& t = buf[(cur + 1) % 4];
        Tensor& sc = buf[(cur + 2) % 4];
        Tensor& o = buf[(cur + 3) % 4];
        // blob order within a block: conv a, conv b, projection
        const size_t at_a = at, at_b = at_a + (size_t)width * bc_in * 9,
                     at_p = at_b + (size_t)width * width * 9;
        at = at_p + (proj ? (size_t)width * bc_in : 0);
        t.pitch = width;
        const Tensor* shortcut = &a;
        if (proj) {
          // the projection reads the centre-tap pixels of conv a: one kernel computes both
          sc.pitch = width;
          bool fused = false;
          conv_layer(a, at_a, width, 3, 2, 1, true, nullptr, &t, false, false, at_p, &sc, &fused);
          if (!fused) conv_layer(a, at_p, width, 1, 2, 0, false, nullptr, &sc, false, false);
          shortcut = &sc;
        } else if (width == 64 && block64_fits(d, a)) {
          // the whole block in one launch; the intermediate tensor t is never written
          o.pitch = width;
          block64_layer(a, at_a, at_b, &o);
          cur = (cur + 3) % 4;
          cin = width;
          continue;
        } else {
          conv_layer(a, at_a, width, 3, 1, 1, true, nullptr, &t, false, false);
        }
        const bool last = s == 3 && blk == 1;
        if (last) { o.p = concat; o.pitch = 768; } else { o.pitch = width; }
        conv_layer(t, at_b, width, 3, 1, 1, true, shortcut, &o, false, false);
        cur = (cur + 3) % 4;
        cin = width;
      }
    }
    Tensor cat;
    cat.p = concat; cat.h = hf; cat.w = wf; cat.c = 768; cat.pitch = 768;
    Tensor gates;
    const int lstm_conv = conv_layer(cat, at, 1024, 3, 1, 1, false, nullptr, &gates, false, true);
    lstm_conv_op = lstm_conv;
    at += (size_t)1024 * 768 * 9;
    // head weights: 8 x 256 fp16, plain [k][c]; the head runs inside the ConvLSTM epilogue
    const size_t w_off = reserve_w(2048);
    if (pack)
      for (int i = 0; i < 2048; ++i) host_w[w_off + i] = (f16)blob[at + i];
    at += 2048;
    {
      Op op;
      op.fam = F_LSTM;
      op.lstm = LstmEpilogueParams{nullptr, ops[lstm_conv].conv.nsplit, mf, 256, cstate,
                                   concat ? concat + 512 : nullptr, 768,
                                   d_w ? d_w + w_off : nullptr, nullptr, hf * wf};
      op.bytes = (double)ops[lstm_conv].conv.nsplit * mf * 1024 * 4.0 + (double)mf * 256 * 10.0;
      op.flops = 2.0 * mf * 8 * 256;
      ops.push_back(op);
      logits_op = (int)ops.size() - 1;
    }
    blob_off = at;
    map_h = hf; map_w = wf; stateful = true;
    d_c = cstate; d_concat = concat;
  }

  void walk(int ph, int pw) {
    if (d.net == HS_NET_TINY4) walk_tiny(ph, pw); else walk_resnet(ph, pw);
  }
};

static void padded_input_geometry(int net_w, int net_h, int k, int* pw, int* ph, int* pad) {
  const int p = k / 2, chunk_px = (k <= 4) ? 4 : 8;
  const int wout = conv_out(net_w, k, 2, p);
  *pad = p;
  *ph = net_h + 2 * p;
  *pw = round_up(std::max(net_w + 2 * p, 2 * (wout - 1) + chunk_px), 2);
}

static size_t expected_weight_floats(int net) {
  if (net == HS_NET_TINY4) return 16 * 3 * 9 + 32 * 16 * 9 + 32 * 32 * 9 + 8 * 32 * 9;
  size_t n = 64 * 3 * 49;
  int cin = 64;
  const int widths[4] = {64, 128, 256, 512};
  for (int s = 0; s < 4; ++s) {
    const int w = widths[s];
    n += (size_t)w * cin * 9 + (size_t)w * w * 9 * 3;
    if (cin != w) n += (size_t)w * cin;
    cin = w;
  }
  n += (size_t)1024 * 768 * 9 + 8 * 256;
  return n;
}

static hs_status validate_desc(const hs_app_desc* d) {
  if (!d) { set_error("NULL description"); return HS_E_INVAL; }
  if (d->frame_w < 1 || d->frame_h < 1 || d->net_w < 8 || d->net_h < 8 || d->frame_w > 10922 ||
      d->frame_h > 65535 || d->net_w > 16384 || d->net_h > 16384) {
    set_error("bad frame or network size");
    return HS_E_INVAL;
  }
  if (d->frame_pitch < (size_t)3 * d->frame_w || d->frame_pitch % 16 != 0) {
    set_error("frame_pitch must be >= 3*frame_w and a multiple of 16");
    return HS_E_INVAL;
  }
  // exact 32-bit integer resize: 255*D + D/2 with D = 4*net_w*net_h must stay below 2^31
  if ((double)d->net_w * d->net_h * 4.0 * 255.5 >= 2147483648.0 ||
      (2.0 * d->net_w + 1.0) * d->frame_w >= 2147483648.0 ||
      (2.0 * d->net_h + 1.0) * d->frame_h >= 2147483648.0) {
    set_error("resize dimensions exceed the exact 32-bit range");
    return HS_E_INVAL;
  }
  if (d->net != HS_NET_TINY4 && d->net != HS_NET_RESNET18_CONVLSTM) {
    set_error("unknown network kind %d", d->net);
    return HS_E_INVAL;
  }
  if (!std::isfinite(d->mean) || !(d->std > 0.0f) || !std::isfinite(d->std) ||
      !(d->threshold > 0.0f && d->threshold < 1.0f) || !(d->alpha >= 0.0f && d->alpha <= 1.0f)) {
    set_error("mean must be finite, std finite and > 0, threshold in (0,1), alpha in [0,1]");
    return HS_E_INVAL;
  }
  if (d->annotate && (d->marker_arm < 0 || d->marker_arm > 64 || d->marker_half < 0 ||
                      d->marker_half > 8 || d->glyph_scale < 1 || d->glyph_scale > 8)) {
    set_error("annotation: marker_arm 0..64, marker_half 0..8, glyph_scale 1..8");
    return HS_E_INVAL;
  }
  if (d->batch < 1 || d->batch > 16) {
    set_error("batch must be 1..16");
    return HS_E_INVAL;
  }
  if (d->queue_depth < 1 || d->queue_depth > 64) {
    set_error("queue_depth must be 1..64");
    return HS_E_INVAL;
  }
  return HS_OK;
}

// Builds the whole plan into `app`, or only sizes the workspace when app == NULL.
static hs_status build_plan(const hs_app_desc* d, hs_app* app, size_t* bytes_out) {
  const bool create = app != nullptr;
  const int depth = d->queue_depth;
  const int k1 = d->net == HS_NET_TINY4 ? 3 : 7;
  int pw, ph, pad;
  padded_input_geometry(d->net_w, d->net_h, k1, &pw, &ph, &pad);

  // sizing walk: packed-weight size
  Builder sizing(*d, nullptr, false, false);
  sizing.walk(ph, pw);
  if (sizing.blob_off != expected_weight_floats(d->net)) {
    set_error("internal: layer walk consumed %zu floats, expected %zu", sizing.blob_off,
              expected_weight_floats(d->net));
    return HS_E_INVAL;
  }

  // real walk: workspace = [weights][activations, state][split-K scratch][tables][slots]
  Builder b(*d, create ? d->d_workspace : nullptr, create, true);
  b.d_w = b.carve.take<f16>(sizing.w_halves);
  b.walk(ph, pw);
  auto bind_partial = [](Builder& bb) {
    float* d_partial = bb.carve.take<float>(bb.partial_floats);
    bb.d_partial = d_partial;
    for (Op& op : bb.ops) {
      if (op.fam == F_CONV && op.conv.use_partial) {
        op.conv.partial = d_partial;
        if (op.conv.wt2)
          op.conv.partial2 = d_partial + (size_t)op.conv.nsplit * op.conv.m * op.conv.cout_pad;
      }
      if (op.fam == F_SPLITK) {
        op.splitk.partial = d_partial;
        if (op.splitk.out2)
          op.splitk.partial2 =
              d_partial + (size_t)op.splitk.nsplit * op.splitk.m * op.splitk.cout_pad;
      }
      if (op.fam == F_LSTM) op.lstm.partial = d_partial;
    }
  };
  bind_partial(b);
  // Further lanes: the same plan over their own activations and scratch (weights shared), so
  // that consecutive frames can overlap.  Slot i runs in lane i % lanes and frames must rotate
  // strictly, hence lanes divides the queue depth.  The cell state c is shared; a lane's state
  // update writes h where the NEXT lane's gate convolution reads it.
  const int lanes = depth % kMaxLanes == 0 ? kMaxLanes : 1;
  std::vector<std::unique_ptr<Builder>> extra;
  std::vector<Builder*> lane_b{&b};
  for (int l = 1; l < lanes; ++l) {
    extra.emplace_back(new Builder(*d, create ? d->d_workspace : nullptr, false, true));
    Builder& bl = *extra.back();
    bl.carve.off = lane_b.back()->carve.off;
    bl.d_w = b.d_w;
    bl.walk(ph, pw);
    bind_partial(bl);
    lane_b.push_back(&bl);
  }
  if (lanes > 1) {
    b.carve.off = lane_b.back()->carve.off;
    if (b.stateful) {
      std::vector<f16*> own_h(lanes);
      for (int l = 0; l < lanes; ++l) own_h[l] = lane_b[l]->ops[b.logits_op].lstm.h_out;
      for (int l = 0; l < lanes; ++l) {
        LstmEpilogueParams& ll = lane_b[l]->ops[b.logits_op].lstm;
        ll.c = b.ops[b.logits_op].lstm.c;
        ll.h_out = own_h[(l + 1) % lanes];
      }
    }
  }
  float* d_lut32 = b.carve.take<float>(256);
  f16* d_lut16 = b.carve.take<f16>(256);
  const int mh = b.map_h, mw = b.map_w;
  const size_t n_map = (size_t)mh * mw;
  const int B = d->batch;
  struct SlotBuf { f16* netin; float* netin32; float* logits; float* heat; uint8_t* mask;
                   uint8_t* kmap; int* marks; };
  std::vector<SlotBuf> sb(depth);
  for (int i = 0; i < depth; ++i) {
    sb[i].netin = b.carve.take<f16>((size_t)B * ph * pw * 4);
    sb[i].netin32 = d->net_fp32_input ? b.carve.take<float>((size_t)B * 3 * d->net_h * d->net_w)
                                      : nullptr;
    sb[i].logits = b.carve.take<float>(B * 8 * n_map);
    sb[i].heat = b.carve.take<float>(B * 8 * n_map);
    sb[i].mask = b.carve.take<uint8_t>(B * 8 * n_map);
    sb[i].kmap = b.carve.take<uint8_t>(B * n_map);
    sb[i].marks = d->annotate ? b.carve.take<int>((size_t)B * 16) : nullptr;
  }
  const size_t total = round_up_sz(b.carve.off, 256);
  if (bytes_out) *bytes_out = total;
  if (!create) return HS_OK;

  if (d->workspace_bytes < total) {
    set_error("workspace too small: %zu bytes given, %zu needed", d->workspace_bytes, total);
    return HS_E_NOMEM;
  }
  app->map_h = mh; app->map_w = mw; app->stateful = b.stateful; app->batch = B;
  app->d_c = b.d_c; app->concat_pitch = 768; app->hid = 256;
  for (int l = 0; l < lanes; ++l) app->d_concat[l] = lane_b[l]->d_concat;
  app->lanes = lanes;
  app->x_ch = 512;

  // upload weights and tables, zero the recurrent state and the padded borders
  HS_HIP(hipMemcpy(b.d_w, b.host_w.data(), b.host_w.size() * sizeof(f16), hipMemcpyHostToDevice));
  {
    float lut32[256];
    f16 lut16[256];
    for (int v = 0; v < 256; ++v) {
      lut32[v] = (float)(((double)v / 255.0 - (double)d->mean) / (double)d->std);
      lut16[v] = (f16)lut32[v];
    }
    HS_HIP(hipMemcpy(d_lut32, lut32, sizeof(lut32), hipMemcpyHostToDevice));
    HS_HIP(hipMemcpy(d_lut16, lut16, sizeof(lut16), hipMemcpyHostToDevice));
  }
  for (int i = 0; i < depth; ++i)
    HS_HIP(hipMemset(sb[i].netin, 0, (size_t)B * ph * pw * 4 * sizeof(f16)));
  if (app->stateful) {
    HS_HIP(hipMemset(app->d_c, 0, B * n_map * 256 * sizeof(float)));
    for (int l = 0; l < lanes; ++l)
      HS_HIP(hipMemset(app->d_concat[l], 0, B * n_map * 768 * sizeof(f16)));
  }
  HS_HIP(hipDeviceSynchronize());

  // per-slot launch plans
  app->netin_w = pw; app->netin_h = ph; app->netin_pad = pad;
  const double theta_d = std::log((double)d->threshold / (1.0 - (double)d->threshold));
  int a_q8 = (int)lrint(256.0 * (double)d->alpha);
  a_q8 = std::max(0, std::min(256, a_q8));
  HS_HIP(hipHostMalloc(&app->pinned, sizeof(PostRecord) * depth * B, hipHostMallocDefault));
  std::memset(app->pinned, 0, sizeof(PostRecord) * depth * B);
  app->slots.resize(depth);
  for (int i = 0; i < depth; ++i) {
    Slot& s = app->slots[i];
    s.d_netin = sb[i].netin; s.d_netin_f32 = sb[i].netin32;
    s.d_logits = sb[i].logits; s.d_heat = sb[i].heat; s.d_mask = sb[i].mask;
    s.rec = (PostRecord*)app->pinned + (size_t)i * B;
    s.results.resize(B);
    {
      Op r;
      r.fam = F_RESIZE;
      ResizeParams& rp = r.resize;
      std::memset(&rp, 0, sizeof(rp));
      rp.batch = B; rp.src_pitch = d->frame_pitch;
      rp.dst_img_stride = (size_t)ph * pw * 4;
      rp.dst32_img_stride = (size_t)3 * d->net_h * d->net_w;
      rp.wi = d->frame_w; rp.hi = d->frame_h; rp.wo = d->net_w; rp.ho = d->net_h;
      rp.dst = s.d_netin; rp.dst_w = pw; rp.pad_l = pad; rp.pad_t = pad;
      rp.dst_f32 = s.d_netin_f32; rp.lut32 = d_lut32; rp.lut16 = d_lut16;
      rp.rcp_dx = 1.0f / (2.0f * d->net_w); rp.rcp_dy = 1.0f / (2.0f * d->net_h);
      {
        // D = 4*wo*ho; l = ceil(log2 D); magic = ceil(2^(31+l) / D) < 2^32.  The error term
        // magic*D - 2^(31+l) is below D <= 2^l, so floor(n/D) = (n*magic) >> (31+l) for n < 2^31.
        const uint64_t D = 4ull * (uint64_t)d->net_w * (uint64_t)d->net_h;
        int l = 0;
        while ((1ull << l) < D) ++l;
        const unsigned __int128 num = (unsigned __int128)1 << (31 + l);
        rp.d_magic = (uint32_t)((num + D - 1) / D);
        rp.d_shift = (uint32_t)(l - 1);
      }
      // algorithmic bytes: the frame read once, three fp16 channels written per pixel (the
      // fourth, zero channel of the padded layout is this implementation's, not the method's)
      r.bytes = B * (3.0 * d->frame_w * d->frame_h + 6.0 * d->net_w * d->net_h +
                     (d->net_fp32_input ? 12.0 * d->net_w * d->net_h : 0.0));
      s.pre.push_back(r);
    }
    s.lane = i % lanes;
    s.infer = lane_b[s.lane]->ops;
    if (b.stateful) { s.wait_idx = b.lstm_conv_op; s.record_idx = b.logits_op; }
    if (s.infer[b.first_conv_op].fam == F_STEM) s.infer[b.first_conv_op].stem.in = s.d_netin;
    else s.infer[b.first_conv_op].conv.in = s.d_netin;
    Op& lo = s.infer[b.logits_op];
    if (lo.fam == F_CONV) lo.conv.out_f32 = s.d_logits;
    else if (lo.fam == F_SPLITK) lo.splitk.out_f32 = s.d_logits;
    else lo.lstm.logits = s.d_logits;
    app->partial_bytes = b.partial_floats * sizeof(float);
    if (app->partial_bytes <= app->ctx->static_scratch_bytes && app->ctx->d_static_scratch) {
      // the same launches with every split-K pointer moved from the lane's scratch in the
      // workspace to the same offset inside the library's fixed array
      float* const from = lane_b[s.lane]->d_partial;
      float* const to = (float*)app->ctx->d_static_scratch;
      auto move = [&](auto*& ptr) {
        if (ptr) ptr = to + (ptr - from);
      };
      s.infer_static = s.infer;
      for (Op& op : s.infer_static) {
        if (op.fam == F_CONV) { move(op.conv.partial); move(op.conv.partial2); }
        if (op.fam == F_SPLITK) { move(op.splitk.partial); move(op.splitk.partial2); }
        if (op.fam == F_LSTM) move(op.lstm.partial);
      }
    }
    {
      Op p;
      p.fam = F_POST;
      p.post = PostParams{s.d_logits, (int)n_map, (float)theta_d, s.d_heat, s.d_mask, s.rec, B,
                          sb[i].kmap, sb[i].marks, mw, mh, d->frame_w, d->frame_h};
      p.bytes = B * 8.0 * n_map * (4 + 4 + 1);
      s.post.push_back(p);
    }
    {
      Op o;
      o.fam = F_OVERLAY;
      OverlayParams& op = o.overlay;
      std::memset(&op, 0, sizeof(op));
      op.batch = B; op.pitch = d->frame_pitch;
      op.wf = d->frame_w; op.hf = d->frame_h;
      op.rcp_gpr = 1.0f / (float)((d->frame_w + 15) / 16);
      op.rcp_hf = 1.0f / (float)d->frame_h; op.rcp_wf = 1.0f / (float)d->frame_w;
      op.n_layers = 1;
      OverlayLayer& L = op.layer[0];
      L.kmap = sb[i].kmap; L.wm = mw; L.hm = mh;
      L.rcp_wm = 1.0f / (float)mw;
      L.a = a_q8;
      L.marks = sb[i].marks;
      L.arm = d->marker_arm; L.half = d->marker_half; L.scale = d->glyph_scale;
      L.rcp_scale = 1.0f / (float)std::max(1, d->glyph_scale);
      for (int g = 0; g < 9; ++g) {
        uint64_t bits = 0;
        for (int r = 0; r < 7; ++r)
          for (int c = 0; c < 5; ++c)
            if ((d->glyphs[g][r] >> (4 - c)) & 1) bits |= 1ull << (5 * r + c);
        L.glyph[g] = bits;
      }
      for (int k = 0; k < 8; ++k)
        L.pal[k] = (uint32_t)d->palette[k][0] | ((uint32_t)d->palette[k][1] << 8) |
                   ((uint32_t)d->palette[k][2] << 16);
      o.bytes = B * (6.0 * d->frame_w * d->frame_h + 1.0 * n_map);
      s.overlay.push_back(o);
    }
    HS_HIP(hipEventCreate(&s.ev_pre));
    HS_HIP(hipEventCreate(&s.ev_infer));
    HS_HIP(hipEventCreate(&s.ev_post));
    HS_HIP(hipEventCreate(&s.ev_overlay));
    HS_HIP(hipEventCreate(&s.ev_state));
  }
  return HS_OK;
}

// ---- completion thread ---------------------------------------------------------------------------
static void completer_main(hs_app* app) {
  (void)hipSetDevice(app->ctx->device);
  for (;;) {
    Slot* s = nullptr;
    {
      std::unique_lock<std::mutex> lk(app->mu);
      app->cv_work.wait(lk, [&] { return app->stop || app->n_completed < app->n_submitted; });
      if (app->n_completed >= app->n_submitted) return;   // stop requested and nothing pending
      s = &app->slots[app->n_completed % app->depth];
    }
    hipError_t e = hipEventSynchronize(s->ev_overlay);
    const uint64_t t_done = now_ns();
    float ms_pre = 0, ms_inf = 0, ms_post = 0;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms_pre, s->ev_pre, s->ev_overlay);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms_inf, s->ev_infer, s->ev_overlay);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms_post, s->ev_post, s->ev_overlay);
    auto back = [&](float ms) {
      const double ns = (double)ms * 1e6;
      return t_done - (uint64_t)std::max(0.0, ns);
    };
    for (size_t j = 0; j < s->results.size(); ++j) {
      hs_result& r = s->results[j];
      r.t_overlay_done_ns = t_done;
      r.t_pre_done_ns = back(ms_pre);
      r.t_infer_done_ns = back(ms_inf);
      r.t_post_done_ns = back(ms_post);
      std::memcpy(r.argmax_idx, s->rec[j].argmax_idx, sizeof(r.argmax_idx));
      std::memcpy(r.peak, s->rec[j].peak, sizeof(r.peak));
      std::memcpy(r.present, s->rec[j].present, sizeof(r.present));
    }
    {
      std::lock_guard<std::mutex> lk(app->mu);
      if (e != hipSuccess && app->completer_error.empty())
        app->completer_error = hipGetErrorString(e);
      s->state = SLOT_DONE;
      app->n_completed++;
    }
    app->cv_done.notify_all();
  }
}

static void destroy_streams(hs_app* app) {
  if (app->s_overlay && app->s_overlay != app->s_lane[0]) (void)hipStreamDestroy(app->s_overlay);
  for (int l = kMaxLanes - 1; l >= 0; --l)
    if (app->s_lane[l] && (l == 0 || app->s_lane[l] != app->s_lane[0]))
      (void)hipStreamDestroy(app->s_lane[l]);
  for (int l = 0; l < kMaxLanes; ++l) app->s_lane[l] = nullptr;
  app->s_overlay = nullptr;
}

static hs_status make_streams(hs_app* app, const uint32_t* mi, const uint32_t* mo, int n_words) {
  hipStream_t sl[kMaxLanes] = {nullptr};
  hipStream_t so = nullptr;
  hipError_t e = hipSuccess;
  if (mi && std::memcmp(mi, mo, sizeof(uint32_t) * (size_t)n_words) == 0) {
    // equal masks: one stream, i.e. one hardware queue, carries all four stages of every lane
    e = hipExtStreamCreateWithCUMask(&sl[0], (uint32_t)n_words, mi);
    so = sl[0];
  } else if (mi) {
    e = hipExtStreamCreateWithCUMask(&sl[0], (uint32_t)n_words, mi);
    if (e == hipSuccess) e = hipExtStreamCreateWithCUMask(&so, (uint32_t)n_words, mo);
  } else if (app->lanes > 1) {
    // the overlay follows its frame's stream (the lanes already overlap one frame's overlay
    // with the next frame's first stages): lanes streams per application, no more
    for (int l = 0; l < app->lanes && e == hipSuccess; ++l)
      e = hipStreamCreateWithFlags(&sl[l], hipStreamNonBlocking);
  } else {
    e = hipStreamCreateWithFlags(&sl[0], hipStreamNonBlocking);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&so, hipStreamNonBlocking);
  }
  if (e != hipSuccess) {
    for (int l = 0; l < kMaxLanes; ++l)
      if (sl[l]) (void)hipStreamDestroy(sl[l]);
    if (so && so != sl[0]) (void)hipStreamDestroy(so);
    set_error("creating the application's streams failed: %s", hipGetErrorString(e));
    return HS_E_DEVICE;
  }
  for (int l = 1; l < kMaxLanes; ++l)
    if (!sl[l]) sl[l] = sl[0];   // partitioned, or fewer lanes: in one queue, in order
  destroy_streams(app);
  for (int l = 0; l < kMaxLanes; ++l) {
    app->s_lane[l] = sl[l];
    app->lane_last_stream[l] = nullptr;   // no frame is in flight here
  }
  app->s_overlay = so;
  return HS_OK;
}

static bool frames_in_flight(hs_app* app) {
  std::lock_guard<std::mutex> lk(app->mu);
  return app->n_completed < app->n_submitted;
}

static void collect_timing(hs_app* app) {
  for (TimedLaunch& t : app->timed) {
    float ms = 0;
    if (hipEventSynchronize(t.e1) == hipSuccess && hipEventElapsedTime(&ms, t.e0, t.e1) == hipSuccess) {
      app->acc_ms[t.fam] += ms;
      app->acc_flops[t.fam] += t.flops;
      app->acc_bytes[t.fam] += t.bytes;
      app->acc_n[t.fam] += 1;
    }
    (void)hipEventDestroy(t.e0);
    (void)hipEventDestroy(t.e1);
  }
  app->timed.clear();
}

static hs_status run_ops(hs_app* app, std::vector<Op>& ops, hipStream_t st, size_t first = 0,
                         size_t last = (size_t)-1) {
  for (size_t i = first; i < std::min(last, ops.size()); ++i) {
    Op& op = ops[i];
    if (app->timing) {
      TimedLaunch t{op.fam, op.flops, op.bytes, nullptr, nullptr};
      HS_HIP(hipEventCreate(&t.e0));
      HS_HIP(hipEventCreate(&t.e1));
      // events attached to the dispatch itself: elapsed = the kernel's own begin -> end
      // time stamps, without the gap between consecutive dispatches
      const KernelDesc d = op_desc(op);
      void* args[1] = {op_params(op)};
      HS_HIP(hipExtLaunchKernel(d.func, d.grid, d.block, args, d.shmem, st, t.e0, t.e1, 0));
      app->timed.push_back(t);
    } else {
      HS_HIP(launch_op(op, st));
    }
  }
  return HS_OK;
}

static hipKernelNodeParams node_params(Op& op, void** args) {
  const KernelDesc d = op_desc(op);
  hipKernelNodeParams kp;
  std::memset(&kp, 0, sizeof(kp));
  kp.func = const_cast<void*>(d.func);
  kp.gridDim = d.grid;
  kp.blockDim = d.block;
  kp.sharedMemBytes = d.shmem;
  args[0] = op_params(op);
  kp.kernelParams = args;
  kp.extra = nullptr;
  return kp;
}

// Stages 1-3 of one queue slot as a linear HIP graph: resize, [event], network kernels,
// [event], postprocess.  Built once; per frame only the resize node's source pointer changes.
// wait_ev: the previous slot's ev_state (the frame before this slot's frame ran there).
static hs_status build_slot_graph(Slot& s, hipEvent_t wait_ev) {
  HS_HIP(hipGraphCreate(&s.graph, 0));
  hipGraphNode_t prev = nullptr;
  auto add_kernel = [&](Op& op, hipGraphNode_t* out) -> hipError_t {
    void* args[1];
    hipKernelNodeParams kp = node_params(op, args);
    hipGraphNode_t n = nullptr;
    hipError_t e = hipGraphAddKernelNode(&n, s.graph, prev ? &prev : nullptr, prev ? 1 : 0, &kp);
    prev = n;
    if (out) *out = n;
    return e;
  };
  auto add_event = [&](hipEvent_t ev) -> hipError_t {
    hipGraphNode_t n = nullptr;
    hipError_t e = hipGraphAddEventRecordNode(&n, s.graph, &prev, 1, ev);
    prev = n;
    return e;
  };
  s.resize_nodes.resize(s.pre.size());
  for (size_t j = 0; j < s.pre.size(); ++j) HS_HIP(add_kernel(s.pre[j], &s.resize_nodes[j]));
  HS_HIP(add_event(s.ev_pre));
  for (size_t j = 0; j < s.infer.size(); ++j) {
    if ((int)j == s.wait_idx && wait_ev) {
      hipGraphNode_t n = nullptr;
      HS_HIP(hipGraphAddEventWaitNode(&n, s.graph, &prev, 1, wait_ev));
      prev = n;
    }
    HS_HIP(add_kernel(s.infer[j], nullptr));
    if ((int)j == s.record_idx) HS_HIP(add_event(s.ev_state));
  }
  HS_HIP(add_event(s.ev_infer));
  for (Op& op : s.post) HS_HIP(add_kernel(op, nullptr));
  HS_HIP(hipGraphInstantiate(&s.graph_exec, s.graph, nullptr, nullptr, 0));
  return HS_OK;
}

}  // namespace hs

// ================================================================================================
// No C++ exception may cross the C boundary: calls that allocate host memory or start threads
// run inside this guard.
template <class F>
static hs_status guarded(const char* fn, F&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    hs::set_error("%s: out of host memory", fn);
    return HS_E_NOMEM;
  } catch (const std::exception& e) {
    hs::set_error("%s: %s", fn, e.what());
    return HS_E_DEVICE;
  }
}

extern "C" {

}  // extern "C"

int hs_internal_app_batch(const hs_app* app) { return app->batch; }
int hs_internal_app_grouped(const hs_app* app) { return app->group != nullptr; }

extern "C" {

hs_status hs_init(int device, hs_ctx** out) {
  if (!out) { set_error("hs_init: NULL out"); return HS_E_INVAL; }
  *out = nullptr;
  int n = 0;
  hipError_t e = hipGetDeviceCount(&n);
  if (e != hipSuccess || device < 0 || device >= n) {
    set_error("hs_init: no HIP device %d (%s)", device,
              e == hipSuccess ? "out of range" : hipGetErrorString(e));
    return HS_E_DEVICE;
  }
  HS_HIP(hipSetDevice(device));
  hipDeviceProp_t prop;
  HS_HIP(hipGetDeviceProperties(&prop, device));
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
    set_error("hs_init: device %d is %s; this library contains gfx950 code only", device,
              prop.gcnArchName);
    return HS_E_DEVICE;
  }
  // the fixed scratch array of this device (for hs_submit_frame_static_scratch)
  void* d_scratch = nullptr;
  size_t scratch_bytes = 0;
  HS_HIP(static_scratch_address(&d_scratch, &scratch_bytes));
  hs_ctx* c = new hs_ctx();
  c->device = device;
  c->n_cus = prop.multiProcessorCount;
  c->d_static_scratch = d_scratch;
  c->static_scratch_bytes = scratch_bytes;
  *out = c;
  return HS_OK;
}

hs_status hs_shutdown(hs_ctx* ctx) {
  if (!ctx) { set_error("hs_shutdown: NULL"); return HS_E_INVAL; }
  {
    std::lock_guard<std::mutex> lk(ctx->mu);
    if (!ctx->apps.empty()) {
      set_error("hs_shutdown: %zu applications still exist", ctx->apps.size());
      return HS_E_STATE;
    }
  }
  delete ctx;
  return HS_OK;
}

hs_status hs_device_cus(hs_ctx* ctx, int* n_cus) {
  if (!ctx || !n_cus) { set_error("hs_device_cus: NULL"); return HS_E_INVAL; }
  *n_cus = ctx->n_cus;
  return HS_OK;
}

hs_status hs_device_copy(hs_ctx* ctx, void* d_dst, const void* d_src, size_t bytes) {
  if (!ctx || !d_dst || !d_src || bytes % 16 != 0 || ((uintptr_t)d_dst & 15) || ((uintptr_t)d_src & 15)) {
    set_error("hs_device_copy: NULL, misaligned pointer or size not a multiple of 16");
    return HS_E_INVAL;
  }
  HS_HIP(hipSetDevice(ctx->device));
  launch_copy(d_dst, d_src, bytes, nullptr);
  HS_HIP(hipGetLastError());
  HS_HIP(hipStreamSynchronize(nullptr));
  return HS_OK;
}

hs_status hs_partition_copy(hs_app* app, void* d_dst, const void* d_src, size_t bytes,
                            int repeats, double* seconds_per_copy) {
  if (!app || !d_dst || !d_src || !seconds_per_copy || repeats < 1 || bytes == 0 ||
      bytes % 16 != 0 || ((uintptr_t)d_dst & 15) || ((uintptr_t)d_src & 15)) {
    set_error("hs_partition_copy: NULL, misaligned pointer, size not a multiple of 16 or repeats < 1");
    return HS_E_INVAL;
  }
  if (frames_in_flight(app)) { set_error("hs_partition_copy: frames in flight"); return HS_E_STATE; }
  HS_HIP(hipSetDevice(app->ctx->device));
  hipStream_t st = app->s_overlay ? app->s_overlay : app->s_lane[0];
  hipEvent_t e0 = nullptr, e1 = nullptr;
  HS_HIP(hipEventCreate(&e0));
  hipError_t e = hipEventCreate(&e1);
  if (e == hipSuccess) {
    launch_copy(d_dst, d_src, bytes, st);   // untimed: first touch of the buffers
    e = hipEventRecord(e0, st);
  }
  for (int i = 0; i < repeats && e == hipSuccess; ++i) {
    launch_copy(d_dst, d_src, bytes, st);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipEventRecord(e1, st);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (e != hipSuccess) {
    set_error("hs_partition_copy: %s", hipGetErrorString(e));
    return HS_E_DEVICE;
  }
  *seconds_per_copy = (double)ms * 1e-3 / repeats;
  return HS_OK;
}

hs_status hs_query_workspace(const hs_app_desc* desc, size_t* bytes) {
  return guarded("hs_query_workspace", [&]() -> hs_status {
  if (!bytes) { set_error("hs_query_workspace: NULL bytes"); return HS_E_INVAL; }
  hs_status st = validate_desc(desc);
  if (st != HS_OK) return st;
  return build_plan(desc, nullptr, bytes);
  });
}

hs_status hs_create_app(hs_ctx* ctx, const hs_app_desc* desc, hs_app** out) {
  return guarded("hs_create_app", [&]() -> hs_status {
  if (!ctx || !out) { set_error("hs_create_app: NULL argument"); return HS_E_INVAL; }
  *out = nullptr;
  hs_status st = validate_desc(desc);
  if (st != HS_OK) return st;
  if (!desc->weights || desc->weight_floats != expected_weight_floats(desc->net)) {
    set_error("weight blob has %zu floats, network needs %zu", desc->weights ? desc->weight_floats : 0,
              expected_weight_floats(desc->net));
    return HS_E_INVAL;
  }
  if (!desc->d_workspace || ((uintptr_t)desc->d_workspace & 255) != 0) {
    set_error("d_workspace must be a 256-byte aligned device pointer");
    return HS_E_INVAL;
  }
  HS_HIP(hipSetDevice(ctx->device));
  hs_app* app = new (std::nothrow) hs_app();
  if (!app) { set_error("hs_create_app: out of host memory"); return HS_E_NOMEM; }
  app->ctx = ctx;
  app->desc = *desc;
  app->desc.weights = nullptr;   // not retained
  app->depth = desc->queue_depth;
  size_t need = 0;
  st = build_plan(desc, app, &need);
  for (size_t i = 0; st == HS_OK && i < app->slots.size(); ++i) {
    const size_t n_slots = app->slots.size();
    st = build_slot_graph(app->slots[i],
                          n_slots > 1 ? app->slots[(i + n_slots - 1) % n_slots].ev_state : nullptr);
  }
  if (st == HS_OK) st = make_streams(app, nullptr, nullptr, 0);
  if (st != HS_OK) {
    for (Slot& s : app->slots) {
      if (s.graph_exec) (void)hipGraphExecDestroy(s.graph_exec);
      if (s.graph) (void)hipGraphDestroy(s.graph);
      if (s.ev_pre) (void)hipEventDestroy(s.ev_pre);
      if (s.ev_infer) (void)hipEventDestroy(s.ev_infer);
      if (s.ev_post) (void)hipEventDestroy(s.ev_post);
      if (s.ev_overlay) (void)hipEventDestroy(s.ev_overlay);
      if (s.ev_state) (void)hipEventDestroy(s.ev_state);
    }
    destroy_streams(app);
    if (app->pinned) (void)hipHostFree(app->pinned);
    delete app;
    return st;
  }
  app->completer = std::thread(completer_main, app);
  {
    std::lock_guard<std::mutex> lk(ctx->mu);
    ctx->apps.push_back(app);
  }
  *out = app;
  return HS_OK;
  });
}

hs_status hs_destroy_app(hs_app* app) {
  if (!app) { set_error("hs_destroy_app: NULL"); return HS_E_INVAL; }
  if (app->group) { set_error("hs_destroy_app: destroy the application's group first"); return HS_E_STATE; }
  (void)hipSetDevice(app->ctx->device);
  {
    std::lock_guard<std::mutex> lk(app->mu);
    app->stop = true;
  }
  app->cv_work.notify_all();
  if (app->completer.joinable()) app->completer.join();   // drains pending frames first
  for (int l = 0; l < kMaxLanes; ++l)
    if (app->s_lane[l]) (void)hipStreamSynchronize(app->s_lane[l]);
  if (app->s_overlay) (void)hipStreamSynchronize(app->s_overlay);
  collect_timing(app);
  for (Slot& s : app->slots) {
    if (s.graph_exec) (void)hipGraphExecDestroy(s.graph_exec);
    if (s.graph) (void)hipGraphDestroy(s.graph);
    (void)hipEventDestroy(s.ev_pre);
    (void)hipEventDestroy(s.ev_infer);
    (void)hipEventDestroy(s.ev_post);
    (void)hipEventDestroy(s.ev_overlay);
    (void)hipEventDestroy(s.ev_state);
  }
  destroy_streams(app);
  if (app->pinned) (void)hipHostFree(app->pinned);
  {
    std::lock_guard<std::mutex> lk(app->ctx->mu);
    auto& v = app->ctx->apps;
    v.erase(std::remove(v.begin(), v.end(), app), v.end());
  }
  delete app;
  return HS_OK;
}

// Lane the most recently submitted frame ran in (0 before the first frame).
static int last_frame_lane(hs_app* app) {
  std::lock_guard<std::mutex> lk(app->mu);
  if (app->n_submitted == 0) return app->lanes - 1;   // so that the "next" lane is lane 0
  return app->slots[(app->n_submitted - 1) % app->depth].lane;
}

hs_status hs_reset_state(hs_app* app) {
  if (!app) { set_error("hs_reset_state: NULL"); return HS_E_INVAL; }
  if (frames_in_flight(app)) { set_error("hs_reset_state: frames in flight"); return HS_E_STATE; }
  if (!app->stateful) return HS_OK;
  HS_HIP(hipSetDevice(app->ctx->device));
  const size_t n = (size_t)app->map_w * app->map_h * app->batch;
  launch_fill_zero(app->d_c, n * app->hid * sizeof(float), app->s_lane[0]);
  for (int l = 0; l < app->lanes; ++l)
    launch_fill_zero(app->d_concat[l], n * app->concat_pitch * sizeof(f16), app->s_lane[0]);
  HS_HIP(hipGetLastError());
  HS_HIP(hipStreamSynchronize(app->s_lane[0]));
  return HS_OK;
}

hs_status hs_get_state(hs_app* app, int stream, float* h_out, float* c_out) {
  if (!app) { set_error("hs_get_state: NULL"); return HS_E_INVAL; }
  if (!app->stateful) { set_error("hs_get_state: network has no recurrent state"); return HS_E_INVAL; }
  if (stream < 0 || stream >= app->batch) { set_error("hs_get_state: no stream %d", stream); return HS_E_INVAL; }
  if (frames_in_flight(app)) { set_error("hs_get_state: frames in flight"); return HS_E_STATE; }
  HS_HIP(hipSetDevice(app->ctx->device));
  const size_t n = (size_t)app->map_w * app->map_h;
  const int hid = app->hid;
  if (c_out) {
    std::vector<float> tmp(n * hid);
    HS_HIP(hipMemcpy(tmp.data(), app->d_c + (size_t)stream * n * hid, tmp.size() * sizeof(float),
                     hipMemcpyDeviceToHost));
    for (size_t m = 0; m < n; ++m)
      for (int j = 0; j < hid; ++j) c_out[(size_t)j * n + m] = tmp[m * hid + j];
  }
  if (h_out) {
    // h of the last frame sits where the NEXT frame's gate convolution will read it
    const f16* cat = app->d_concat[(last_frame_lane(app) + 1) % app->lanes];
    std::vector<f16> tmp(n * app->concat_pitch);
    HS_HIP(hipMemcpy(tmp.data(), cat + (size_t)stream * n * app->concat_pitch,
                     tmp.size() * sizeof(f16), hipMemcpyDeviceToHost));
    for (size_t m = 0; m < n; ++m)
      for (int j = 0; j < hid; ++j)
        h_out[(size_t)j * n + m] = (float)tmp[m * app->concat_pitch + app->x_ch + j];
  }
  return HS_OK;
}

hs_status hs_get_features(hs_app* app, int stream, float* x_out) {
  if (!app || !x_out) { set_error("hs_get_features: NULL"); return HS_E_INVAL; }
  if (!app->stateful) { set_error("hs_get_features: network has no recurrent cell"); return HS_E_INVAL; }
  if (stream < 0 || stream >= app->batch) { set_error("hs_get_features: no stream %d", stream); return HS_E_INVAL; }
  if (frames_in_flight(app)) { set_error("hs_get_features: frames in flight"); return HS_E_STATE; }
  HS_HIP(hipSetDevice(app->ctx->device));
  const size_t n = (size_t)app->map_w * app->map_h;
  std::vector<f16> tmp(n * app->concat_pitch);
  const f16* cat = app->d_concat[last_frame_lane(app)];
  HS_HIP(hipMemcpy(tmp.data(), cat + (size_t)stream * n * app->concat_pitch,
                   tmp.size() * sizeof(f16), hipMemcpyDeviceToHost));
  for (size_t m = 0; m < n; ++m)
    for (int j = 0; j < app->x_ch; ++j)
      x_out[(size_t)j * n + m] = (float)tmp[m * app->concat_pitch + j];
  return HS_OK;
}

hs_status hs_set_partition(hs_app* app, const uint32_t* cu_mask_infer,
                           const uint32_t* cu_mask_overlay, int n_words) {
  return guarded("hs_set_partition", [&]() -> hs_status {
  if (!app) { set_error("hs_set_partition: NULL app"); return HS_E_INVAL; }
  if ((cu_mask_infer == nullptr) != (cu_mask_overlay == nullptr)) {
    set_error("hs_set_partition: give both masks or neither");
    return HS_E_INVAL;
  }
  if (frames_in_flight(app)) { set_error("hs_set_partition: frames in flight"); return HS_E_STATE; }
  hs_ctx* ctx = app->ctx;
  HS_HIP(hipSetDevice(ctx->device));
  std::lock_guard<std::mutex> lk(ctx->mu);
  if (!cu_mask_infer) {
    hs_status st = make_streams(app, nullptr, nullptr, 0);
    if (st != HS_OK) return st;
    std::memset(app->claim, 0, sizeof(app->claim));
    app->partitioned = false;
    return HS_OK;
  }
  uint32_t others[HS_MAX_CU_WORDS] = {0};
  for (hs_app* o : ctx->apps)
    if (o != app)
      for (int w = 0; w < HS_MAX_CU_WORDS; ++w) others[w] |= o->claim[w];
  hs_status st = admission_check(others, cu_mask_infer, cu_mask_overlay, n_words, ctx->n_cus);
  if (st != HS_OK) return st;
  st = make_streams(app, cu_mask_infer, cu_mask_overlay, n_words);
  if (st != HS_OK) return st;
  std::memset(app->claim, 0, sizeof(app->claim));
  for (int w = 0; w < n_words; ++w) app->claim[w] = cu_mask_infer[w] | cu_mask_overlay[w];
  app->partitioned = true;
  return HS_OK;
  });
}

// Marks the slot as in flight and wakes the completion thread (the last step of a submit).
static void finish_submit(hs_app* app, Slot* s) {
  const uint64_t t_enq = now_ns();
  for (hs_result& r : s->results) r.t_enqueued_ns = t_enq;
  {
    std::lock_guard<std::mutex> lk(app->mu);
    s->state = SLOT_INFLIGHT;
    app->n_submitted++;
  }
  app->cv_work.notify_one();
}

// Enqueues stages 1-3 of one batch and, with own_overlay, stage 4 as well.  Without it the
// caller draws the overlay (a group), records s->ev_overlay and calls finish_submit; *slot_out
// and *stream_out then name the slot taken and the stream whose tail is the ev_post record.
static hs_status enqueue_stages(hs_app* app, Slot* s, bool idle, const uint8_t* const* d_frames,
                                uint8_t* const* d_overlay_outs, uint64_t frame_id,
                                uint64_t t_submit, bool own_overlay, Slot** slot_out,
                                hipStream_t* stream_out, hipEvent_t frames_ready,
                                bool static_scratch);

// A submit that fails after part of a frame has been handed to the GPU leaves the recurrent
// state advanced by a frame that is never delivered: the application is unusable from then on.
// Every later submit returns HS_E_DEVICE with this message.
static void poison(hs_app* app, const char* what) {
  std::lock_guard<std::mutex> lk(app->mu);
  if (app->completer_error.empty())
    app->completer_error = std::string("a submit failed after work had been enqueued (") + what +
                           "); destroy the application";
}

static hs_status submit_stages(hs_app* app, const uint8_t* const* d_frames,
                               uint8_t* const* d_overlay_outs, uint64_t frame_id,
                               uint64_t t_submit, bool own_overlay, Slot** slot_out,
                               hipStream_t* stream_out, hipEvent_t frames_ready = nullptr,
                               bool static_scratch = false) {
  if (!app || !d_frames || !d_overlay_outs) { set_error("hs_submit_batch: NULL argument"); return HS_E_INVAL; }
  const int B = app->batch;
  for (int j = 0; j < B; ++j) {
    if (!d_frames[j] || !d_overlay_outs[j]) { set_error("hs_submit_batch: NULL frame pointer"); return HS_E_INVAL; }
    if (((uintptr_t)d_frames[j] & 15) || ((uintptr_t)d_overlay_outs[j] & 15)) {
      set_error("hs_submit_batch: frame pointers must be 16-byte aligned");
      return HS_E_INVAL;
    }
    if (d_frames[j] == d_overlay_outs[j]) { set_error("hs_submit_batch: output aliases input"); return HS_E_INVAL; }
  }
  Slot* s = nullptr;
  bool idle = false;   // nothing in flight: this frame cannot overlap with an earlier one
  {
    std::lock_guard<std::mutex> lk(app->mu);
    if (!app->completer_error.empty()) {
      set_error("device error in an earlier frame: %s", app->completer_error.c_str());
      return HS_E_DEVICE;
    }
    if (app->n_submitted - app->n_delivered >= (uint64_t)app->depth) {
      set_error("hs_submit_batch: queue full (%d slots)", app->depth);
      return HS_E_QUEUE_FULL;
    }
    s = &app->slots[app->n_submitted % app->depth];
    idle = app->n_completed == app->n_submitted;
    if (static_scratch && !idle) {
      // one scratch array serves every frame that uses it: no second frame beside it
      set_error("hs_submit_frame_static_scratch: a frame of this application is still in flight");
      return HS_E_STATE;
    }
  }
  const hs_status st = enqueue_stages(app, s, idle, d_frames, d_overlay_outs, frame_id, t_submit,
                                      own_overlay, slot_out, stream_out, frames_ready,
                                      static_scratch);
  if (st != HS_OK) poison(app, hs_last_error());
  return st;
}

static hs_status enqueue_stages(hs_app* app, Slot* s, bool idle, const uint8_t* const* d_frames,
                                uint8_t* const* d_overlay_outs, uint64_t frame_id,
                                uint64_t t_submit, bool own_overlay, Slot** slot_out,
                                hipStream_t* stream_out, hipEvent_t frames_ready,
                                bool static_scratch) {
  HS_HIP(hipSetDevice(app->ctx->device));
  std::vector<Op>& infer = static_scratch ? s->infer_static : s->infer;
  const int B = app->batch;
  const size_t n_map = (size_t)app->map_w * app->map_h;
  const size_t netin_img = (size_t)app->netin_h * app->netin_w * 4;
  for (int j = 0; j < B; ++j) {
    hs_result& r = s->results[j];
    std::memset(&r, 0, sizeof(r));
    r.frame_id = frame_id;
    r.t_submit_ns = t_submit;
    r.map_w = app->map_w; r.map_h = app->map_h;
    r.net_input_pitch_bytes = (size_t)app->netin_w * 4 * sizeof(f16);
    r.d_overlay = d_overlay_outs[j];
    r.d_mask = s->d_mask + j * 8 * n_map;
    r.d_heat = s->d_heat + j * 8 * n_map;
    r.d_logits = s->d_logits + j * 8 * n_map;
    r.d_net_input = s->d_netin + j * netin_img +
                    ((size_t)app->netin_pad * app->netin_w + app->netin_pad) * 4;
    r.d_net_input_f32 = s->d_netin_f32
                            ? s->d_netin_f32 + (size_t)j * 3 * app->desc.net_h * app->desc.net_w
                            : nullptr;
    s->pre[0].resize.src[j] = d_frames[j];
    s->overlay[0].overlay.src[j] = d_frames[j];
    s->overlay[0].overlay.dst[j] = d_overlay_outs[j];
  }

  hs_status st = HS_OK;
  // A frame that finds the application idle runs on the first stream whatever its lane (paced
  // streams then use one queue, like a single-lane application); otherwise on its lane's stream,
  // behind the lane's previous frame if that one ran elsewhere (they share activation buffers).
  hipStream_t lane_stream = idle ? app->s_lane[0] : app->s_lane[s->lane];
  if (!idle && app->lane_last_stream[s->lane] && app->lane_last_stream[s->lane] != lane_stream &&
      app->depth >= app->lanes) {
    Slot& same_lane =
        app->slots[(size_t)((s - app->slots.data()) + app->depth - app->lanes) % app->depth];
    HS_HIP(hipStreamWaitEvent(lane_stream, same_lane.ev_post, 0));
  }
  app->lane_last_stream[s->lane] = lane_stream;
  // the caller's producer (another stream) may still be writing the frames
  if (frames_ready) HS_HIP(hipStreamWaitEvent(lane_stream, frames_ready, 0));
  if (app->launch_mode == HS_LAUNCH_GRAPH && !app->timing && !static_scratch) {
    void* args[1];
    hipKernelNodeParams kp = node_params(s->pre[0], args);
    HS_HIP(hipGraphExecKernelNodeSetParams(s->graph_exec, s->resize_nodes[0], &kp));
    HS_HIP(hipGraphLaunch(s->graph_exec, lane_stream));
  } else {
    st = run_ops(app, s->pre, lane_stream);
    if (st != HS_OK) return st;
    HS_HIP(hipEventRecord(s->ev_pre, lane_stream));
    if (s->wait_idx >= 0) {
      // the recurrent cell waits for the previous frame's state update (other lane)
      Slot& before = app->slots[(size_t)((s - app->slots.data()) + app->depth - 1) % app->depth];
      st = run_ops(app, infer, lane_stream, 0, (size_t)s->wait_idx);
      if (st != HS_OK) return st;
      if (app->depth > 1) HS_HIP(hipStreamWaitEvent(lane_stream, before.ev_state, 0));
      st = run_ops(app, infer, lane_stream, (size_t)s->wait_idx, (size_t)s->record_idx + 1);
      if (st != HS_OK) return st;
      HS_HIP(hipEventRecord(s->ev_state, lane_stream));
      st = run_ops(app, infer, lane_stream, (size_t)s->record_idx + 1);
    } else {
      st = run_ops(app, infer, lane_stream);
    }
    if (st != HS_OK) return st;
    HS_HIP(hipEventRecord(s->ev_infer, lane_stream));
    st = run_ops(app, s->post, lane_stream);
    if (st != HS_OK) return st;
  }
  HS_HIP(hipEventRecord(s->ev_post, lane_stream));
  if (!own_overlay) {
    *slot_out = s;
    *stream_out = lane_stream;
    return HS_OK;
  }
  hipStream_t ov_stream = app->s_overlay ? app->s_overlay : lane_stream;
  if (ov_stream != lane_stream) HS_HIP(hipStreamWaitEvent(ov_stream, s->ev_post, 0));
  st = run_ops(app, s->overlay, ov_stream);
  if (st != HS_OK) return st;
  HS_HIP(hipEventRecord(s->ev_overlay, ov_stream));
  finish_submit(app, s);
  return HS_OK;
}

static hs_status refuse_grouped(hs_app* app, const char* fn) {
  if (app && app->group) {
    set_error("%s: the application is a member of a group; use the hs_*_group calls", fn);
    return HS_E_STATE;
  }
  return HS_OK;
}

hs_status hs_submit_batch(hs_app* app, const uint8_t* const* d_frames,
                          uint8_t* const* d_overlay_outs, uint64_t frame_id) {
  const uint64_t t_submit = now_ns();
  if (refuse_grouped(app, "hs_submit_batch") != HS_OK) return HS_E_STATE;
  return submit_stages(app, d_frames, d_overlay_outs, frame_id, t_submit, true, nullptr, nullptr);
}

hs_status hs_submit_batch_after(hs_app* app, const uint8_t* const* d_frames,
                                uint8_t* const* d_overlay_outs, uint64_t frame_id,
                                void* hip_event_frames_ready) {
  const uint64_t t_submit = now_ns();
  if (refuse_grouped(app, "hs_submit_batch_after") != HS_OK) return HS_E_STATE;
  return submit_stages(app, d_frames, d_overlay_outs, frame_id, t_submit, true, nullptr, nullptr,
                       (hipEvent_t)hip_event_frames_ready);
}

hs_status hs_submit_frame(hs_app* app, const uint8_t* d_frame, uint8_t* d_overlay_out,
                          uint64_t frame_id) {
  if (!app) { set_error("hs_submit_frame: NULL argument"); return HS_E_INVAL; }
  if (app->batch != 1) {
    set_error("hs_submit_frame: the application batches %d streams; use hs_submit_batch", app->batch);
    return HS_E_STATE;
  }
  return hs_submit_batch(app, &d_frame, &d_overlay_out, frame_id);
}

hs_status hs_submit_frame_static_scratch(hs_app* app, const uint8_t* d_frame,
                                         uint8_t* d_overlay_out, uint64_t frame_id) {
  const uint64_t t_submit = now_ns();
  if (!app) { set_error("hs_submit_frame_static_scratch: NULL argument"); return HS_E_INVAL; }
  if (refuse_grouped(app, "hs_submit_frame_static_scratch") != HS_OK) return HS_E_STATE;
  if (app->batch != 1) {
    set_error("hs_submit_frame_static_scratch: the application batches %d streams", app->batch);
    return HS_E_STATE;
  }
  if (app->timing) {   // per-kernel timing creates events, i.e. allocates
    set_error("hs_submit_frame_static_scratch: kernel timing is on");
    return HS_E_STATE;
  }
  if (app->slots[0].infer_static.empty()) {
    set_error("hs_submit_frame_static_scratch: a frame of this application needs %zu bytes of "
              "split-K scratch, the library's fixed array holds %zu", app->partial_bytes,
              app->ctx->static_scratch_bytes);
    return HS_E_NOMEM;
  }
  return submit_stages(app, &d_frame, &d_overlay_out, frame_id, t_submit, true, nullptr, nullptr,
                       nullptr, true);
}

// Copies the oldest finished batch's results (one per stream) out and frees its slot.
static hs_status deliver_locked(hs_app* app, hs_result* out) {
  Slot& s = app->slots[app->n_delivered % app->depth];
  const uint64_t t_obs = now_ns();
  for (size_t j = 0; j < s.results.size(); ++j) {
    out[j] = s.results[j];
    out[j].t_observed_ns = t_obs;
  }
  s.state = SLOT_FREE;
  app->n_delivered++;
  if (!app->completer_error.empty()) {
    set_error("device error: %s", app->completer_error.c_str());
    return HS_E_DEVICE;
  }
  return HS_OK;
}

hs_status hs_poll_batch(hs_app* app, hs_result* out) {
  if (!app || !out) { set_error("hs_poll_batch: NULL argument"); return HS_E_INVAL; }
  if (refuse_grouped(app, "hs_poll_batch") != HS_OK) return HS_E_STATE;
  std::lock_guard<std::mutex> lk(app->mu);
  if (app->n_delivered >= app->n_completed) {
    set_error("hs_poll_batch: no finished frame");
    return HS_E_NOT_READY;
  }
  return deliver_locked(app, out);
}

hs_status hs_wait_batch(hs_app* app, hs_result* out, uint64_t timeout_ns) {
  if (!app || !out) { set_error("hs_wait_batch: NULL argument"); return HS_E_INVAL; }
  if (refuse_grouped(app, "hs_wait_batch") != HS_OK) return HS_E_STATE;
  std::unique_lock<std::mutex> lk(app->mu);
  const bool ok = app->cv_done.wait_for(lk, std::chrono::nanoseconds(timeout_ns), [&] {
    return app->n_delivered < app->n_completed;
  });
  if (!ok) {
    set_error("hs_wait_batch: timed out");
    return HS_E_NOT_READY;
  }
  return deliver_locked(app, out);
}

hs_status hs_poll_result(hs_app* app, hs_result* out) {
  if (app && app->batch != 1) {
    set_error("hs_poll_result: the application batches %d streams; use hs_poll_batch", app->batch);
    return HS_E_STATE;
  }
  return hs_poll_batch(app, out);
}

hs_status hs_wait_result(hs_app* app, hs_result* out, uint64_t timeout_ns) {
  if (app && app->batch != 1) {
    set_error("hs_wait_result: the application batches %d streams; use hs_wait_batch", app->batch);
    return HS_E_STATE;
  }
  return hs_wait_batch(app, out, timeout_ns);
}

// ---- multi-network applications ---------------------------------------------------------------
static_assert(HS_MAX_GROUP == kMaxLayers, "one overlay layer per group member");

static void group_worker_main(GroupWorker* w, int device) {
  (void)hipSetDevice(device);
  for (;;) {
    {
      std::unique_lock<std::mutex> lk(w->mu);
      w->cv.wait(lk, [&] { return w->has_job || w->stop; });
      if (!w->has_job) return;
      w->has_job = false;
    }
    const hs_status st = submit_stages(w->app, &w->d_frame, &w->d_out, w->frame_id, w->t_submit,
                                       false, &w->slot, &w->tail);
    {
      std::lock_guard<std::mutex> lk(w->mu);
      w->status = st;
      if (st != HS_OK) w->error = hs_last_error();
      w->done = true;
    }
    w->cv.notify_all();
  }
}

hs_status hs_create_group(hs_ctx* ctx, hs_app* const* members, int n_members, hs_group** out) {
  return guarded("hs_create_group", [&]() -> hs_status {
  if (!ctx || !members || !out) { set_error("hs_create_group: NULL argument"); return HS_E_INVAL; }
  if (n_members < 1 || n_members > kMaxLayers) {
    set_error("hs_create_group: %d members, 1..%d allowed", n_members, kMaxLayers);
    return HS_E_INVAL;
  }
  for (int i = 0; i < n_members; ++i) {
    hs_app* a = members[i];
    if (!a || a->ctx != ctx) { set_error("hs_create_group: member %d is NULL or of another context", i); return HS_E_INVAL; }
    for (int j = 0; j < i; ++j)
      if (members[j] == a) { set_error("hs_create_group: member %d listed twice", i); return HS_E_INVAL; }
    if (a->batch != 1) { set_error("hs_create_group: member %d batches %d streams", i, a->batch); return HS_E_INVAL; }
    const hs_app_desc &d = a->desc, &d0 = members[0]->desc;
    if (d.frame_w != d0.frame_w || d.frame_h != d0.frame_h || d.frame_pitch != d0.frame_pitch) {
      set_error("hs_create_group: member %d takes another frame geometry than member 0", i);
      return HS_E_INVAL;
    }
    if (a->group) { set_error("hs_create_group: member %d already belongs to a group", i); return HS_E_STATE; }
    std::lock_guard<std::mutex> lk(a->mu);
    if (a->n_delivered != a->n_submitted) {
      set_error("hs_create_group: member %d has frames in flight or unpolled", i);
      return HS_E_STATE;
    }
  }
  hs_group* g = new (std::nothrow) hs_group();
  if (!g) { set_error("hs_create_group: out of host memory"); return HS_E_NOMEM; }
  g->ctx = ctx;
  g->members.assign(members, members + n_members);
  // the frame-level fields of the overlay launch come from member 0; layers are set per frame
  Op o = members[0]->slots[0].overlay[0];
  o.overlay.n_layers = n_members;
  double map_bytes = 0;
  for (hs_app* a : g->members) map_bytes += (double)a->map_w * a->map_h;
  o.bytes = 6.0 * members[0]->desc.frame_w * members[0]->desc.frame_h + map_bytes;
  g->overlay.push_back(o);
  for (int i = 1; i < n_members; ++i) {
    g->workers.emplace_back(new GroupWorker());
    GroupWorker* w = g->workers.back().get();
    w->app = members[i];
    w->th = std::thread(group_worker_main, w, ctx->device);
  }
  for (hs_app* a : g->members) a->group = g;
  *out = g;
  return HS_OK;
  });
}

hs_status hs_destroy_group(hs_group* group) {
  if (!group) { set_error("hs_destroy_group: NULL"); return HS_E_INVAL; }
  for (hs_app* a : group->members) {   // frames in flight still need the group's bookkeeping
    std::unique_lock<std::mutex> lk(a->mu);
    a->cv_done.wait(lk, [&] { return a->n_completed == a->n_submitted; });
  }
  for (auto& w : group->workers) {
    {
      std::lock_guard<std::mutex> lk(w->mu);
      w->stop = true;
    }
    w->cv.notify_all();
    w->th.join();
  }
  for (hs_app* a : group->members) a->group = nullptr;
  delete group;
  return HS_OK;
}

hs_status hs_submit_group(hs_group* group, const uint8_t* d_frame, uint8_t* d_overlay_out,
                          uint64_t frame_id) {
  const uint64_t t_submit = now_ns();
  if (!group || !d_frame || !d_overlay_out) { set_error("hs_submit_group: NULL argument"); return HS_E_INVAL; }
  const size_t n = group->members.size();
  // nothing is enqueued unless every member can take the frame
  for (size_t i = 0; i < n; ++i) {
    hs_app* a = group->members[i];
    std::lock_guard<std::mutex> lk(a->mu);
    if (!a->completer_error.empty()) {
      set_error("device error in an earlier frame: %s", a->completer_error.c_str());
      return HS_E_DEVICE;
    }
    if (a->n_submitted - a->n_delivered >= (uint64_t)a->depth) {
      set_error("hs_submit_group: queue of member %d full (%d slots)", (int)i, a->depth);
      return HS_E_QUEUE_FULL;
    }
  }
  Slot* slot[kMaxLayers];
  hipStream_t tail[kMaxLayers];
  OverlayParams& op = group->overlay[0].overlay;
  for (auto& w : group->workers) {   // members 1.. on their own threads
    {
      std::lock_guard<std::mutex> lk(w->mu);
      w->d_frame = d_frame; w->d_out = d_overlay_out;
      w->frame_id = frame_id; w->t_submit = t_submit;
      w->done = false;
      w->has_job = true;
    }
    w->cv.notify_all();
  }
  hs_status st0 = submit_stages(group->members[0], &d_frame, &d_overlay_out, frame_id, t_submit,
                                false, &slot[0], &tail[0]);
  std::string err0 = st0 != HS_OK ? hs_last_error() : "";
  for (size_t i = 1; i < n; ++i) {   // always collect every worker, also after a failure
    GroupWorker* w = group->workers[i - 1].get();
    std::unique_lock<std::mutex> lk(w->mu);
    w->cv.wait(lk, [&] { return w->done; });
    slot[i] = w->slot; tail[i] = w->tail;
    if (st0 == HS_OK && w->status != HS_OK) { st0 = w->status; err0 = w->error; }
  }
  // From here on a failure leaves some members a frame ahead of the others (their cells have
  // been updated by a frame that will never be delivered): the whole group is poisoned.
  auto fail_all = [&](hs_status st) {
    const std::string why = hs_last_error();
    for (hs_app* a : group->members) poison(a, why.c_str());
    set_error("%s", why.c_str());
    return st;
  };
  if (st0 != HS_OK) { set_error("%s", err0.c_str()); return fail_all(st0); }
  for (size_t i = 0; i < n; ++i) op.layer[i] = slot[i]->overlay[0].overlay.layer[0];
  op.src[0] = d_frame;
  op.dst[0] = d_overlay_out;
  // one launch draws every member's layer, on member 0's overlay stream, after all stage 3s
  hs_app* a0 = group->members[0];
  hipStream_t ov_stream = a0->s_overlay ? a0->s_overlay : tail[0];
  auto overlay_all = [&]() -> hs_status {
    for (size_t i = 0; i < n; ++i)
      if (tail[i] != ov_stream) HS_HIP(hipStreamWaitEvent(ov_stream, slot[i]->ev_post, 0));
    const hs_status st = run_ops(a0, group->overlay, ov_stream);
    if (st != HS_OK) return st;
    for (size_t i = 0; i < n; ++i) HS_HIP(hipEventRecord(slot[i]->ev_overlay, ov_stream));
    return HS_OK;
  };
  const hs_status st = overlay_all();
  if (st != HS_OK) return fail_all(st);
  for (size_t i = 0; i < n; ++i) finish_submit(group->members[i], slot[i]);
  return HS_OK;
}

// Delivers one frame's results of all members if every member has finished it.
static hs_status deliver_group(hs_group* group, hs_result* out) {
  for (hs_app* a : group->members) {
    std::lock_guard<std::mutex> lk(a->mu);
    if (a->n_delivered >= a->n_completed) {
      set_error("hs_poll_group: no finished frame");
      return HS_E_NOT_READY;
    }
  }
  hs_status worst = HS_OK;
  for (size_t i = 0; i < group->members.size(); ++i) {
    hs_app* a = group->members[i];
    std::lock_guard<std::mutex> lk(a->mu);
    const hs_status st = deliver_locked(a, out + i);
    if (st != HS_OK) worst = st;
  }
  return worst;
}

hs_status hs_poll_group(hs_group* group, hs_result* out) {
  if (!group || !out) { set_error("hs_poll_group: NULL argument"); return HS_E_INVAL; }
  return deliver_group(group, out);
}

hs_status hs_wait_group(hs_group* group, hs_result* out, uint64_t timeout_ns) {
  if (!group || !out) { set_error("hs_wait_group: NULL argument"); return HS_E_INVAL; }
  const auto deadline = std::chrono::steady_clock::now() + std::chrono::nanoseconds(timeout_ns);
  for (hs_app* a : group->members) {
    std::unique_lock<std::mutex> lk(a->mu);
    if (!a->cv_done.wait_until(lk, deadline, [&] { return a->n_delivered < a->n_completed; })) {
      set_error("hs_wait_group: timed out");
      return HS_E_NOT_READY;
    }
  }
  return deliver_group(group, out);
}

hs_status hs_set_launch_mode(hs_app* app, int mode) {
  if (!app) { set_error("hs_set_launch_mode: NULL"); return HS_E_INVAL; }
  if (mode != HS_LAUNCH_GRAPH && mode != HS_LAUNCH_EAGER) {
    set_error("hs_set_launch_mode: unknown mode %d", mode);
    return HS_E_INVAL;
  }
  if (frames_in_flight(app)) { set_error("hs_set_launch_mode: frames in flight"); return HS_E_STATE; }
  app->launch_mode = mode;
  return HS_OK;
}

hs_status hs_set_cpu_affinity(hs_app* app, int cpu) {
  if (!app) { set_error("hs_set_cpu_affinity: NULL"); return HS_E_INVAL; }
  cpu_set_t set;
  CPU_ZERO(&set);
  if (cpu < 0) {
    const long n = sysconf(_SC_NPROCESSORS_CONF);
    for (long c = 0; c < n && c < CPU_SETSIZE; ++c) CPU_SET((int)c, &set);
  } else {
    if (cpu >= CPU_SETSIZE) { set_error("hs_set_cpu_affinity: no such core %d", cpu); return HS_E_INVAL; }
    CPU_SET(cpu, &set);
  }
  int rc = pthread_setaffinity_np(app->completer.native_handle(), sizeof(set), &set);
  if (rc == 0 && app->group) {   // a group member's submitting thread follows its completion thread
    const auto& m = app->group->members;
    const size_t i = (size_t)(std::find(m.begin(), m.end(), app) - m.begin());
    if (i >= 1 && i < m.size())
      rc = pthread_setaffinity_np(app->group->workers[i - 1]->th.native_handle(), sizeof(set), &set);
  }
  if (rc != 0) {
    set_error("hs_set_cpu_affinity: core %d refused (%s)", cpu, strerror(rc));
    return HS_E_INVAL;
  }
  return HS_OK;
}

hs_status hs_set_kernel_timing(hs_app* app, int enable) {
  if (!app) { set_error("hs_set_kernel_timing: NULL"); return HS_E_INVAL; }
  if (frames_in_flight(app)) { set_error("hs_set_kernel_timing: frames in flight"); return HS_E_STATE; }
  (void)hipSetDevice(app->ctx->device);
  collect_timing(app);
  for (int f = 0; f < F_COUNT; ++f) {
    app->acc_ms[f] = app->acc_flops[f] = app->acc_bytes[f] = 0;
    app->acc_n[f] = 0;
  }
  app->timing = enable != 0;
  return HS_OK;
}

hs_status hs_get_kernel_times(hs_app* app, hs_kernel_time* entries, int max_entries,
                              int* n_entries) {
  if (!app || !n_entries) { set_error("hs_get_kernel_times: NULL"); return HS_E_INVAL; }
  if (frames_in_flight(app)) { set_error("hs_get_kernel_times: frames in flight"); return HS_E_STATE; }
  (void)hipSetDevice(app->ctx->device);
  collect_timing(app);
  int n = 0;
  for (int f = 0; f < F_COUNT; ++f) {
    if (!app->acc_n[f]) continue;
    if (entries && n < max_entries) {
      hs_kernel_time& k = entries[n];
      std::memset(&k, 0, sizeof(k));
      std::strncpy(k.name, kFamilyName[f], sizeof(k.name) - 1);
      k.launches = app->acc_n[f];
      k.total_ms = app->acc_ms[f];
      k.flops = app->acc_flops[f];
      k.bytes = app->acc_bytes[f];
    }
    ++n;
  }
  *n_entries = n;
  return HS_OK;
}

}  // extern "C"
