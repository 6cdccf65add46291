// C-ABI layer of the slim-attention decode library: argument validation, workspace layout,
// variant choice and kernel sequencing.  No arithmetic of the method lives here.
#include "slim_attention.h"
#include "slim_kernels.h"

#include <math.h>
#include <atomic>
#include <chrono>
#include <mutex>

namespace {

using namespace slim;

constexpr size_t ALIGN = 256;
inline size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

// Scratch layout shared by the decode entry points.  `width` is the row width of the cached
// matrix (d for a K-cache, d_model for an X-cache).
struct Plan {
  int nsplit = 1;      // context splits of the weighted-sum step
  int nsplit_v = 1;    // context splits of the vanilla kernel
  int nsplit_x = 1;    // context splits of the X-cache MFMA path (two passes over X)
  int nsplit_xf = 0;   // context splits of the one-pass X-cache kernel (0: the shape does not take it)
  size_t off_S = 0, off_Cpart = 0, off_m = 0, off_l = 0, off_Cn = 0, off_qt = 0;
  size_t off_vacc = 0, off_vm = 0, off_vl = 0;
  size_t off_exch = 0, off_outpart = 0, off_ctrl = 0;   // bf16 fast path
  bool fused_ok = false;
  FusedGeom geom{};
  int csw = 1;         // row splits of W_KV in the MFMA projection (its own launch)
  int csw_f = 0;       // same, when the stream kernel's workgroups do the projection (0: not possible)
  size_t total = 0;
};

// Control block at the start of every workspace: arrival counters, arrival flags, and in its last two
// ints the id of the latest stream-kernel launch and the error word (= that id when a wait ran out).
constexpr int CTRL_INTS = 4096;

int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

Plan make_plan(int B, int H, int T, int width, int e) {
  Plan p;
  const int ncolblk = (width + 511) / 512, nhb = (H + 31) / 32;
  const long per_split = (long)B * ncolblk * nhb;
  p.nsplit = clampi((int)((1024 + per_split - 1) / per_split), 1, clampi((T + 127) / 128, 1, 64));
  // vanilla kernel: workgroups of four waves, a wave per group of heads; about eight workgroups per
  // compute unit, splits of at least 256 rows
  const int hpw = vanilla_heads_per_wave(DT_BF16, e / H);      // (the packing of the bf16 kernel; harmless for fp32)
  const long per_split_v = (long)B * (((H + (hpw ? hpw : 1) - 1) / (hpw ? hpw : 1) + 3) / 4);
  p.nsplit_v = clampi((int)((2048 + per_split_v - 1) / per_split_v), 1, clampi(T / 256, 1, 256));
  size_t o = 0;
  p.off_ctrl = o;    o += up(sizeof(int) * CTRL_INTS);
  p.fused_ok = (width == e) && fused_geometry(B, H, T, width, &p.geom);
  p.nsplit_x = xcache_splits(B, H, T, width);
  p.nsplit_xf = xfused_ok(width) ? xfused_splits(B, H, T, width) : 0;
  size_t nparts = (size_t)B * (p.nsplit > p.nsplit_x ? p.nsplit : p.nsplit_x);
  if ((size_t)B * p.nsplit_xf > nparts) nparts = (size_t)B * p.nsplit_xf;
  if (p.fused_ok && (size_t)p.geom.nparts > nparts) nparts = p.geom.nparts;
  if (p.fused_ok && (size_t)B * 4 > nparts && fused_by_sequence(p.geom, B, false)) nparts = (size_t)B * 4;
  p.csw = proj_row_splits(H, width, e, B);
  if (p.fused_ok && B <= 16 && p.geom.grid >= H) {
    const int tiles_w = (width + TILE_ROWS - 1) / TILE_ROWS;
    p.csw_f = p.geom.grid / H < tiles_w ? p.geom.grid / H : tiles_w;
  }
  p.off_S = o;      o += up(sizeof(float) * (size_t)B * H * ((T + 31) / 32 * 32));   // (rows padded to 32 scores)
  p.off_Cpart = o;  o += up(sizeof(float) * nparts * H * width);
  p.off_m = o;      o += up(sizeof(float) * nparts * H);
  p.off_l = o;      o += up(sizeof(float) * nparts * H);
  p.off_Cn = o;     o += up(sizeof(float) * (size_t)B * H * width);
  p.off_qt = o;     o += up(sizeof(float) * (size_t)B * ((H + 15) / 16 * 16) * width);   // (whole tiles of 16 heads)
  p.off_vacc = o;   o += up(sizeof(float) * (size_t)B * p.nsplit_v * e);
  p.off_vm = o;     o += up(sizeof(float) * (size_t)B * p.nsplit_v * H);
  p.off_vl = o;     o += up(sizeof(float) * (size_t)B * p.nsplit_v * H);
  if (p.fused_ok) { p.off_exch = o; o += up(fused_exch_bytes(p.geom)); }
  p.off_outpart = o; o += up(sizeof(float) * (size_t)(p.csw > p.csw_f ? p.csw : p.csw_f) * B * e);
  p.total = o;
  return p;
}

// Scratch for callers that may not allocate (slim_decode_static): one array per device, part of the
// loaded code object (set-up also writes its probe result there, so that it needs no allocation).  Host code never uses this name as an address: the address on each device comes
// from hipGetSymbolAddress at set-up (device_state) and is what kernels, copies and queries are given.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)SLIM_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

// Per-device set-up, done once (slim_init, else the first call that needs it) under a lock: the
// address of the static scratch, the compute-unit count, whether workgroup i of a launch runs on XCD
// i % 8 (a probe launch on the null stream and a blocking read-back, no allocation: it writes into
// the static scratch), and the event used to order stream-kernel launches of different streams.
struct DeviceState {
  bool ready = false, xcd_round_robin = false;
  int cus = 0;
  void* static_scratch = nullptr;
  hipEvent_t order_ev = nullptr;
  hipStream_t last_stream = nullptr;
  bool any_launch = false;
  signed char blocks_per_cu[2][2][3] = {};    // [NT - 1][rope][lphp class]: 0 unknown, else 1 + blocks
};
DeviceState g_dev[64];
std::mutex g_dev_mu;

DeviceState* device_state() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) { (void)hipGetLastError(); return nullptr; }
  std::lock_guard<std::mutex> lk(g_dev_mu);
  DeviceState& s = g_dev[dev];
  if (s.ready) return &s;
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return nullptr; }
  s.static_scratch = ptr;
  if (hipDeviceGetAttribute(&s.cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) { (void)hipGetLastError(); s.cus = 0; }
  s.xcd_round_robin = s.cus >= 256 && probe_xcd_round_robin((unsigned*)ptr, nullptr);
  if (hipEventCreateWithFlags(&s.order_ev, hipEventDisableTiming) != hipSuccess) { s.order_ev = nullptr; (void)hipGetLastError(); }
  s.ready = true;
  return &s;
}

// Library-owned scratch: one allocation per device, grown on demand, kept until exit.
struct OwnedScratch { void* ptr = nullptr; size_t bytes = 0; };
OwnedScratch g_scratch[64];
std::mutex g_scratch_mu;

int get_workspace(const slim_opts* o, size_t need, char** ws) {
  if (o && o->workspace) {
    if (o->workspace_bytes < need) return SLIM_ERR_WORKSPACE;
    if (((uintptr_t)o->workspace) & 15) return SLIM_ERR_ALIGN;
    *ws = (char*)o->workspace;
    return SLIM_OK;
  }
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SLIM_ERR_LAUNCH;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  OwnedScratch& s = g_scratch[dev];
  if (s.bytes < need) {
    if (s.ptr) { (void)hipFree(s.ptr); s.ptr = nullptr; s.bytes = 0; }   // hipFree waits for the device
    if (hipMalloc(&s.ptr, need) != hipSuccess) { s.ptr = nullptr; (void)hipGetLastError(); return SLIM_ERR_LAUNCH; }
    s.bytes = need;
  }
  *ws = (char*)s.ptr;
  return SLIM_OK;
}

bool misaligned(const void* p) { return (((uintptr_t)p) & 15) != 0; }

// The stream kernel's workgroups wait for each other, so all of a launch's workgroups must be resident
// together: two such launches running side by side (different streams) could each hold half of the chip
// and starve each other until their waits run out.  Launches that arrive on another stream than the
// previous one are therefore ordered behind it with an event; on one stream this costs nothing.
void order_after_previous_stream_kernel(DeviceState& d, hipStream_t st) {
  std::lock_guard<std::mutex> lk(g_dev_mu);
  if (d.any_launch && d.last_stream != st && d.order_ev) {
    if (hipEventRecord(d.order_ev, d.last_stream) == hipSuccess) (void)hipStreamWaitEvent(st, d.order_ev, 0);
    else (void)hipGetLastError();
  }
  d.last_stream = st;
  d.any_launch = true;
}

// All workgroups of a stream-kernel launch must be resident at once (they wait for each other): the
// device must hold `grid` of them, by its own occupancy figure for this instantiation.
bool stream_kernel_fits(DeviceState& d, const FusedGeom& g, bool rope) {
  const int lc = g.lphp == 16 ? 0 : (g.lphp == 8 ? 1 : 2);
  signed char& slot = d.blocks_per_cu[g.NT - 1][rope ? 1 : 0][lc];
  {
    std::lock_guard<std::mutex> lk(g_dev_mu);
    if (slot == 0) {
      const int n = fused_blocks_per_cu(g, rope);
      slot = (signed char)(1 + (n > 100 ? 100 : (n < 0 ? 0 : n)));
    }
  }
  return (long)(slot - 1) * d.cus >= g.grid;
}

int check_common(int B, int H, int T, int e, int d_k, int width, const slim_opts* o, int* dtype,
                 long* t_stride) {
  if (B < 1 || H < 1 || T < 1 || e < 1 || width < 1) return SLIM_ERR_SHAPE;
  *dtype = o ? o->dtype : SLIM_F32;
  if (*dtype != SLIM_F32 && *dtype != SLIM_BF16) return SLIM_ERR_DTYPE;
  const int vec = vec_elems(*dtype);
  if (d_k < 1 || H * d_k != e) return SLIM_ERR_SHAPE;
  if (d_k % vec != 0 || width % vec != 0) return SLIM_ERR_SHAPE;
  *t_stride = (o && o->t_stride) ? (long)o->t_stride : (long)T;
  if (*t_stride < T) return SLIM_ERR_SHAPE;
  if (o && o->seq_lens && (((uintptr_t)o->seq_lens) & 3)) return SLIM_ERR_ALIGN;
  if (o && o->seq_lens_host)
    for (int b = 0; b < B; ++b)
      if (o->seq_lens_host[b] < 1 || o->seq_lens_host[b] > T) return SLIM_ERR_SEQLEN;
  return SLIM_OK;
}

int launch_status() { return hipGetLastError() == hipSuccess ? SLIM_OK : SLIM_ERR_LAUNCH; }

// Optional per-kernel timing (opts->stage_ms): an event before the first kernel and one after
// each kernel, all on the call's stream; finish() waits for the stream and reads them out.
class StageTimer {
 public:
  StageTimer(const slim_opts* o, hipStream_t st) : out_(o ? o->stage_ms : nullptr), st_(st) {
    if (!out_) return;
    for (int i = 0; i < SLIM_MAX_STAGES; ++i) out_[i] = 0.f;
    for (auto& e : ev_) if (hipEventCreate(&e) != hipSuccess) { out_ = nullptr; return; }
    (void)hipEventRecord(ev_[0], st_);
  }
  void mark() {
    if (out_ && n_ < SLIM_MAX_STAGES) (void)hipEventRecord(ev_[++n_], st_);
  }
  void finish() {
    if (!out_) return;
    (void)hipStreamSynchronize(st_);
    for (int i = 0; i < n_; ++i) (void)hipEventElapsedTime(&out_[i], ev_[i], ev_[i + 1]);
    for (auto& e : ev_) (void)hipEventDestroy(e);
    out_ = nullptr;
  }
 private:
  float* out_;
  hipStream_t st_;
  hipEvent_t ev_[SLIM_MAX_STAGES + 1];
  int n_ = 0;
};

}  // namespace

extern "C" const char* slim_strerror(int code) {
  switch (code) {
    case SLIM_OK: return "ok";
    case SLIM_ERR_ARG: return "null pointer, negative size, or an option this entry point does not take";
    case SLIM_ERR_SHAPE: return "unsupported shape (d % H, d_k vs 16-byte vectors, T, t_stride)";
    case SLIM_ERR_DTYPE: return "dtype must be SLIM_F32 or SLIM_BF16";
    case SLIM_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case SLIM_ERR_WORKSPACE: return "workspace smaller than slim_workspace_bytes()";
    case SLIM_ERR_SINGULAR: return "W_K singular to working precision or non-finite";
    case SLIM_ERR_ILLCOND: return "W_K ill-conditioned (rcond < 1e-12); W_KV written but unreliable";
    case SLIM_ERR_LAUNCH: return "HIP allocation or launch error";
    case SLIM_ERR_SEQLEN: return "sequence length outside [1, T]";
    case SLIM_ERR_LAYOUT: return "banded K-cache: rows per sequence not a multiple of 32, or no kernel reads that layout for this shape / dtype / call";
    case SLIM_ERR_TIMEOUT: return "a wait between workgroups ran out in the latest stream-kernel launch on this workspace; its outputs are NaN";
    default: return "unknown slim status";
  }
}

// The stream kernel's launch geometry is laid out for 256 compute units in 8 XCDs; a device (or
// partition) with fewer takes the plain kernels.  Unknown (no device visible, e.g. when only sizes are
// asked for on a build machine) counts as enough.
bool chip_holds_stream_kernel() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return true; }
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) { (void)hipGetLastError(); return true; }
  return cus >= 256;
}

// Which implementation runs for a K-cache decode of this shape.
int pick_variant(int requested, int B, int H, int T, int d, int dtype) {
  if (requested == SLIM_VARIANT_GENERIC) return SLIM_VARIANT_GENERIC;
  if (!chip_holds_stream_kernel()) return SLIM_VARIANT_GENERIC;
  FusedGeom g;
  const int zb = (B + 15) / 16;                      // upper bound of the projection's batch chunks
  if (dtype == SLIM_BF16 && fused_geometry(B, H, T, d, &g) && H * zb < CTRL_INTS / 2 && g.grid <= CTRL_INTS / 2 - 1)
    return requested == SLIM_VARIANT_FUSED_SPLIT ? SLIM_VARIANT_FUSED_SPLIT : SLIM_VARIANT_FUSED;
  return SLIM_VARIANT_GENERIC;
}

// Tags of the score exchange are unique per launch within the process and start at a random
// point, so words left in a workspace by earlier launches (or an earlier process) never match.
std::atomic<unsigned> g_tag{(unsigned)std::chrono::steady_clock::now().time_since_epoch().count() * 2654435761u};
// Launch ids (arrival flags, error word) start at a random point as well: a fresh workspace may hold
// anything, small integers included.
std::atomic<unsigned> g_launch{((unsigned)std::chrono::steady_clock::now().time_since_epoch().count() * 2246822519u) | 1u};

extern "C" int slim_variant_for(int B, int H, int T, int d, int dtype) {
  if (B < 1 || H < 1 || T < 1 || d < 1 || d % H != 0) return 0;
  if (dtype != SLIM_F32 && dtype != SLIM_BF16) return 0;
  return pick_variant(SLIM_VARIANT_AUTO, B, H, T, d, dtype);
}

extern "C" size_t slim_workspace_bytes(int B, int H, int T, int d, int dtype) {
  if (B < 1 || H < 1 || T < 1 || d < 1) return 0;
  (void)dtype;
  // d is the cached row width; the vanilla partials are sized for e = d (K-cache case).
  return make_plan(B, H, T, d, d).total;
}

extern "C" size_t slim_workspace_bytes_xcache(int B, int H, int T, int d_model, int d_k, int dtype) {
  if (B < 1 || H < 1 || T < 1 || d_model < 1 || d_k < 1) return 0;
  (void)dtype;
  return make_plan(B, H, T, d_model, H * d_k).total;
}

namespace {

// slim_decode and slim_decode_static: the same validation, plan and launches; `fixed_ws` (non-null for
// the static scratch) replaces the workspace lookup.
int decode_core(const void* q, const void* Kcache, const void* W_KV, void* out, int B, int H, int T, int d,
                const slim_opts* o, char* fixed_ws, size_t fixed_ws_bytes) {
  if (!q || !Kcache || !W_KV || !out) return SLIM_ERR_ARG;
  if (H < 1 || d < 1 || d % H != 0) return SLIM_ERR_SHAPE;
  const int d_k = d / H;
  int dtype; long t_stride;
  if (int rc = check_common(B, H, T, d, d_k, d, o, &dtype, &t_stride)) return rc;
  if (misaligned(q) || misaligned(Kcache) || misaligned(W_KV) || misaligned(out)) return SLIM_ERR_ALIGN;
  const float* rope = o ? o->rope_table : nullptr;
  if (rope && (d_k & 1)) return SLIM_ERR_SHAPE;
  if (rope && misaligned(rope)) return SLIM_ERR_ALIGN;
  const Plan p = make_plan(B, H, T, d, d);
  char* ws = fixed_ws;
  if (fixed_ws) {
    if (p.total > fixed_ws_bytes) return SLIM_ERR_WORKSPACE;
  } else if (int rc = get_workspace(o, p.total, &ws)) {
    return rc;
  }
  hipStream_t st = o ? (hipStream_t)o->stream : nullptr;
  const int32_t* lens = o ? o->seq_lens : nullptr;
  const float scale = 1.0f / sqrtf((float)d_k);
  float* S = (float*)(ws + p.off_S);
  float* Cpart = (float*)(ws + p.off_Cpart);
  float* mpart = (float*)(ws + p.off_m);
  float* lpart = (float*)(ws + p.off_l);
  float* Cn = (float*)(ws + p.off_Cn);
  const long kb = t_stride * d;

  StageTimer tm(o, st);
  int variant = pick_variant(o ? o->variant : SLIM_VARIANT_AUTO, B, H, T, d, dtype);
  DeviceState* dev = nullptr;
  if (variant == SLIM_VARIANT_FUSED || variant == SLIM_VARIANT_FUSED_SPLIT) {
    // the stream kernel needs this device's set-up, and all of its workgroups resident together
    dev = device_state();
    if (!dev || !stream_kernel_fits(*dev, p.geom, rope != nullptr)) variant = SLIM_VARIANT_GENERIC;
  }
  const int k_layout = o ? o->k_layout : SLIM_K_ROWMAJOR;
  if (k_layout != SLIM_K_ROWMAJOR && k_layout != SLIM_K_BANDED) return SLIM_ERR_ARG;
  if (k_layout == SLIM_K_BANDED &&
      (t_stride % 32 != 0 || (variant != SLIM_VARIANT_FUSED && variant != SLIM_VARIANT_FUSED_SPLIT)))
    return SLIM_ERR_LAYOUT;                              // only the stream kernel reads banded caches
  if (variant == SLIM_VARIANT_FUSED || variant == SLIM_VARIANT_FUSED_SPLIT) {
    const FusedGeom& g = p.geom;
    int* ctrl = (int*)(ws + p.off_ctrl);
    const int per = 16 * proj_batch_tiles(B, d, d, H);
    const int zb = (B + per - 1) / per;
    FusedArgs fa{};
    fa.q = (const float*)q; fa.K = (const uint16_t*)Kcache; fa.k_bstride = kb; fa.seq_lens = lens;
    fa.k_banded = k_layout == SLIM_K_BANDED;
    fa.T = T; fa.B = B; fa.H = H; fa.d = d; fa.d_k = d_k;
    fa.G = g.G; fa.NG = g.NG; fa.gpx = g.gpx; fa.lph = g.lph; fa.lphp = g.lphp; fa.hpu = g.hpu;
    fa.qscale = scale * 1.4426950408889634f;
    fa.exch = (unsigned long long*)(ws + p.off_exch);
    const unsigned tiles = (unsigned)B * (unsigned)((T + TILE_ROWS - 1) / TILE_ROWS) + (unsigned)B + 64u;
    fa.tag_base = g_tag.fetch_add(tiles);
    unsigned lid = g_launch.fetch_add(1);
    if (lid == 0) lid = g_launch.fetch_add(1);
    fa.launch_id = lid;
    // every wait for another workgroup: 20 ms of real time (100 MHz ticks) unless the caller says otherwise
    const long long budget_us = (o && o->wait_budget_us) ? (long long)o->wait_budget_us : 20000;
    fa.wait_ticks = budget_us < 0 ? 0ull : (unsigned long long)budget_us * 100ull;
    fa.xcd_local = (g.gpx > 0 && dev->xcd_round_robin) ? 1 : 0;
    fa.rope = rope;
    fa.Cpart = Cpart; fa.mpart = mpart; fa.lpart = lpart;
    fa.err = ctrl + CTRL_INTS - 1; fa.counters = ctrl; fa.ncounters = H * zb;
    ProjArgs pa{};
    pa.Cpart = Cpart; pa.mpart = mpart; pa.lpart = lpart; pa.W = (const uint16_t*)W_KV;
    pa.out = (float*)out; pa.outpart = (float*)(ws + p.off_outpart); pa.counters = ctrl;
    pa.err = ctrl + CTRL_INTS - 1; pa.launch_id = lid; pa.seq_lens = lens;
    pa.B = B; pa.T = T; pa.H = H; pa.d_k = d_k; pa.rows = d; pa.e = d;
    pa.NG = g.NG; pa.nsplit = 0; pa.mode = 0; pa.mscale = 1.0f; pa.csw = p.csw;
    if (const int shares = fused_by_sequence(g, B, lens != nullptr)) {
      fa.by_sequence = shares;
      pa.mode = 1; pa.nsplit = shares;               // partials laid out [sequence][share]
    }
    const bool one_launch = variant == SLIM_VARIANT_FUSED && p.csw_f > 0 && !fa.by_sequence;
    if (one_launch) {
      // the stream kernel's workgroups also merge and project (flags after the counters)
      pa.csw = p.csw_f;
      pa.crows = proj_rows_per_split(d, p.csw_f);
      fa.fuse = 1; fa.flags = (unsigned*)(ctrl + CTRL_INTS / 2); fa.proj = pa;
    }
    order_after_previous_stream_kernel(*dev, st);
    launch_fused_stream(g, fa, st);
    tm.mark();
    if (!one_launch) {
      launch_project_mfma(pa, st);
      tm.mark();
    }
    tm.finish();
    return launch_status();
  }
  launch_head_scores(dtype, (const float*)q, d, Kcache, kb, d, lens, T, d, H, d_k, scale, S,
                     (long)H * T, rope, B, st);
  tm.mark();
  launch_weighted_sum(dtype, S, Kcache, kb, d, lens, T, H, p.nsplit, Cpart, mpart, lpart, B, st);
  tm.mark();
  // Shapes the stream kernel does not take (more than 32 heads, very large batches) still get the MFMA
  // merge + projection when the head width allows it; an explicit request for the plain kernels keeps
  // every step on the vector ALU.
  const int requested = o ? o->variant : SLIM_VARIANT_AUTO;
  if (dtype == SLIM_BF16 && requested != SLIM_VARIANT_GENERIC && d_k % 8 == 0 && d_k <= 128 &&
      (long)H * ((B + 15) / 16) < CTRL_INTS / 2) {
    int* ctrl = (int*)(ws + p.off_ctrl);
    launch_zero_ints(ctrl, CTRL_INTS / 2, st);
    ProjArgs pa{};
    pa.Cpart = Cpart; pa.mpart = mpart; pa.lpart = lpart; pa.W = (const uint16_t*)W_KV;
    pa.out = (float*)out; pa.outpart = (float*)(ws + p.off_outpart); pa.counters = ctrl;
    pa.seq_lens = lens; pa.B = B; pa.T = T; pa.H = H; pa.d_k = d_k; pa.rows = d; pa.e = d;
    pa.nsplit = p.nsplit; pa.mode = 1; pa.mscale = 1.4426950408889634f;      // natural-log maxima
    pa.csw = p.csw;
    launch_project_mfma(pa, st);
    tm.mark();
    tm.finish();
    return launch_status();
  }
  launch_combine(Cpart, mpart, lpart, p.nsplit, H, d, Cn, B, st);
  tm.mark();
  launch_project(dtype, Cn, W_KV, d, d, H, d_k, (float*)out, B, st);
  tm.mark();
  tm.finish();
  return launch_status();
}

}  // namespace

extern "C" int slim_decode(const void* q, const void* Kcache, const void* W_KV, void* out, int B,
                           int H, int T, int d, const slim_opts* o) {
  return decode_core(q, Kcache, W_KV, out, B, H, T, d, o, nullptr, 0);
}

extern "C" int slim_init(void) { return device_state() ? SLIM_OK : SLIM_ERR_LAUNCH; }

extern "C" size_t slim_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

extern "C" int slim_decode_static(const void* q, const void* Kcache, const void* W_KV, void* out, int B,
                                  int H, int T, int d, const slim_opts* o) {
  if (o && (o->workspace || o->stage_ms)) return SLIM_ERR_ARG;     // brings its own scratch; timing events allocate
  DeviceState* dev = device_state();
  if (!dev) return SLIM_ERR_LAUNCH;
  return decode_core(q, Kcache, W_KV, out, B, H, T, d, o, (char*)dev->static_scratch, STATIC_SCRATCH_BYTES);
}

extern "C" int slim_status(const void* workspace, void* stream) {
  const char* ws = (const char*)workspace;
  if (workspace == SLIM_STATIC_SCRATCH) {
    DeviceState* dev = device_state();
    if (!dev) return SLIM_ERR_LAUNCH;
    ws = (const char*)dev->static_scratch;
  } else if (!workspace) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) { (void)hipGetLastError(); return SLIM_ERR_LAUNCH; }
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    ws = (const char*)g_scratch[dev].ptr;
    if (!ws) return SLIM_OK;                          // nothing has run on the library's own scratch
  }
  int tail[2] = {0, 0};                               // {id of the latest stream-kernel launch, error word}
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess ||
      hipMemcpy(tail, ws + sizeof(int) * (CTRL_INTS - 2), sizeof(tail), hipMemcpyDeviceToHost) != hipSuccess) {
    (void)hipGetLastError();
    return SLIM_ERR_LAUNCH;
  }
  return (tail[0] != 0 && tail[1] == tail[0]) ? SLIM_ERR_TIMEOUT : SLIM_OK;
}

extern "C" int slim_read_probe(const void* buf, size_t bytes, void* stream) {
  if (!buf || bytes < 16) return SLIM_ERR_ARG;
  if (misaligned(buf)) return SLIM_ERR_ALIGN;
  launch_read_probe(buf, bytes, (hipStream_t)stream);
  return launch_status();
}

extern "C" int vanilla_kv_decode(const void* q, const void* Kcache, const void* Vcache, void* out,
                                 int B, int H, int T, int d, const slim_opts* o) {
  if (!q || !Kcache || !Vcache || !out) return SLIM_ERR_ARG;
  if (o && o->rope_table) return SLIM_ERR_ARG;        // a vanilla cache stores rotated keys
  if (o && o->k_layout) return SLIM_ERR_ARG;          // K and V caches are row-major here
  if (H < 1 || d < 1 || d % H != 0) return SLIM_ERR_SHAPE;
  const int d_k = d / H;
  int dtype; long t_stride;
  if (int rc = check_common(B, H, T, d, d_k, d, o, &dtype, &t_stride)) return rc;
  if (d_k / vec_elems(dtype) > 32) return SLIM_ERR_SHAPE;
  if (misaligned(q) || misaligned(Kcache) || misaligned(Vcache) || misaligned(out)) return SLIM_ERR_ALIGN;
  const Plan p = make_plan(B, H, T, d, d);
  char* ws;
  if (int rc = get_workspace(o, p.total, &ws)) return rc;
  hipStream_t st = o ? (hipStream_t)o->stream : nullptr;
  StageTimer tm(o, st);
  launch_vanilla(dtype, (const float*)q, Kcache, Vcache, t_stride * d, o ? o->seq_lens : nullptr, T,
                 H, d_k, p.nsplit_v, (float*)(ws + p.off_vacc), (float*)(ws + p.off_vm),
                 (float*)(ws + p.off_vl), (float*)out, B, st);
  tm.mark();
  tm.finish();
  return launch_status();
}

extern "C" int slim_decode_xcache(const void* q, const void* X, const void* W_K, const void* W_V,
                                  void* out, int B, int H, int T, int d_model, int d_k,
                                  const slim_opts* o) {
  if (!q || !X || !W_K || !W_V || !out) return SLIM_ERR_ARG;
  if (o && o->rope_table) return SLIM_ERR_ARG;        // no rotary positions in the X-cache scheme
  if (o && o->k_layout) return SLIM_ERR_ARG;          // the X-cache is row-major
  if (H < 1 || d_k < 1 || d_model < 1) return SLIM_ERR_SHAPE;
  const int e = H * d_k;
  int dtype; long t_stride;
  if (int rc = check_common(B, H, T, e, d_k, d_model, o, &dtype, &t_stride)) return rc;
  if (misaligned(q) || misaligned(X) || misaligned(W_K) || misaligned(W_V) || misaligned(out))
    return SLIM_ERR_ALIGN;
  const Plan p = make_plan(B, H, T, d_model, e);
  char* ws;
  if (int rc = get_workspace(o, p.total, &ws)) return rc;
  hipStream_t st = o ? (hipStream_t)o->stream : nullptr;
  const int32_t* lens = o ? o->seq_lens : nullptr;
  const float scale = 1.0f / sqrtf((float)d_k);
  float* S = (float*)(ws + p.off_S);
  float* Cpart = (float*)(ws + p.off_Cpart);
  float* mpart = (float*)(ws + p.off_m);
  float* lpart = (float*)(ws + p.off_l);
  float* Cn = (float*)(ws + p.off_Cn);
  float* qt = (float*)(ws + p.off_qt);
  const long xb = t_stride * d_model;

  StageTimer tm(o, st);
  const int req = o ? o->variant : SLIM_VARIANT_AUTO;
  if (req != SLIM_VARIANT_GENERIC && xcache_fast_ok(dtype, H, d_model, d_k) && H < CTRL_INTS / 2 &&
      (size_t)T * d_model * 2 < ((size_t)1 << 32)) {      // (the kernels address a sequence's rows with 32-bit offsets)
    // MFMA path: q~, scores (log2 domain), weighted sum per context split, merge + projection
    int* ctrl = (int*)(ws + p.off_ctrl);
    const int per = 16 * proj_batch_tiles(B, d_model, e, H);
    const int zb = (B + per - 1) / per;
    launch_xq_tilde((const float*)q, W_K, qt, B, H, d_k, d_model, e, scale * 1.4426950408889634f, ctrl, H * zb, st);
    tm.mark();
    int nsplit = p.nsplit_x;
    if (p.nsplit_xf > 0 && req != SLIM_VARIANT_FUSED_SPLIT) {
      // d_model <= 1024: scores, numerators and weighted sum in one pass over X
      nsplit = p.nsplit_xf;
      launch_xfused(qt, X, xb, lens, T, H, d_model, nsplit, Cpart, mpart, lpart, B, st);
      tm.mark();
    } else {
      launch_xscores(qt, X, xb, lens, T, H, d_model, S, B, st);
      tm.mark();
      launch_xweighted(S, X, xb, lens, T, H, d_model, nsplit, Cpart, mpart, lpart, B, st);
      tm.mark();
    }
    ProjArgs pa{};
    pa.Cpart = Cpart; pa.mpart = mpart; pa.lpart = lpart; pa.W = (const uint16_t*)W_V;
    pa.out = (float*)out; pa.outpart = (float*)(ws + p.off_outpart); pa.counters = ctrl;
    pa.err = nullptr; pa.launch_id = 0; pa.seq_lens = lens;
    pa.B = B; pa.T = T; pa.H = H; pa.d_k = d_k; pa.rows = d_model; pa.e = e;
    pa.NG = 0; pa.nsplit = nsplit; pa.mode = 1; pa.mscale = 1.0f;
    pa.csw = proj_row_splits(H, d_model, e, B);
    launch_project_mfma(pa, st);
    tm.mark();
    tm.finish();
    return launch_status();
  }
  // qt[b][h][c] = sum_j q[b][h d_k + j] W_K[c][h d_k + j]   ("rows" of W_K scored against q)
  launch_head_scores(dtype, (const float*)q, e, W_K, 0, e, nullptr, d_model, e, H, d_k, 1.0f, qt,
                     (long)H * d_model, nullptr, B, st);
  tm.mark();
  launch_dense_scores(dtype, qt, X, xb, d_model, lens, T, H, scale, S, B, st);
  tm.mark();
  launch_weighted_sum(dtype, S, X, xb, d_model, lens, T, H, p.nsplit, Cpart, mpart, lpart, B, st);
  tm.mark();
  launch_combine(Cpart, mpart, lpart, p.nsplit, H, d_model, Cn, B, st);
  tm.mark();
  launch_project(dtype, Cn, W_V, d_model, e, H, d_k, (float*)out, B, st);
  tm.mark();
  tm.finish();
  return launch_status();
}

// ---- the steps either side of the decode step ----------------------------------------------------
namespace {

struct BlockBufs { size_t off_q, off_k, off_v, off_attn, off_dpart, total; };

BlockBufs block_layout(const Plan& p, int B, int H, int d) {
  BlockBufs b;
  size_t o = p.total;
  const size_t row = up(sizeof(float) * (size_t)B * d);
  b.off_q = o; o += row;
  b.off_k = o; o += row;
  b.off_v = o; o += row;
  b.off_attn = o; o += row;
  // partial sums of the dense products: [matrix][row split][B][d] for one, two or three matrices
  size_t parts = 1;
  for (int nmat = 1; nmat <= 3; ++nmat) {
    const size_t n = (size_t)nmat * dense_row_splits(H, nmat, d, d, B);
    if (n > parts) parts = n;
  }
  b.off_dpart = o; o += up(sizeof(float) * parts * B * d);
  b.total = o;
  return b;
}

struct BlockCall {
  const void *x, *W_Q, *W_K, *W_V, *W_second, *W_O;   // W_second: W_KV (slim) or unused (vanilla)
  void *Kcache, *Vcache, *y;
};

int attention_block(bool slim_path, const BlockCall& c, int B, int H, int T, int d, const slim_opts* o) {
  if (!c.x || !c.W_Q || !c.W_K || !c.W_O || !c.Kcache || !c.y) return SLIM_ERR_ARG;
  if (slim_path ? !c.W_second : (!c.W_V || !c.Vcache)) return SLIM_ERR_ARG;
  if (H < 1 || d < 1 || d % H != 0) return SLIM_ERR_SHAPE;
  const int d_k = d / H;
  int dtype; long t_stride;
  if (int rc = check_common(B, H, T, d, d_k, d, o, &dtype, &t_stride)) return rc;
  if (d_k & 1) return SLIM_ERR_SHAPE;
  if (!slim_path && d_k / vec_elems(dtype) > 32) return SLIM_ERR_SHAPE;
  const void* ptrs[] = {c.x, c.W_Q, c.W_K, c.W_V, c.W_second, c.W_O, c.Kcache, c.Vcache, c.y, o ? o->rope_table : nullptr};
  for (const void* q : ptrs) if (q && misaligned(q)) return SLIM_ERR_ALIGN;
  const Plan p = make_plan(B, H, T, d, d);
  const BlockBufs bb = block_layout(p, B, H, d);
  char* ws;
  if (int rc = get_workspace(o, bb.total, &ws)) return rc;
  hipStream_t st = o ? (hipStream_t)o->stream : nullptr;
  const int32_t* lens = o ? o->seq_lens : nullptr;
  const float* rope = o ? o->rope_table : nullptr;
  float* q = (float*)(ws + bb.off_q);
  float* knew = (float*)(ws + bb.off_k);
  float* vnew = (float*)(ws + bb.off_v);
  float* attn = (float*)(ws + bb.off_attn);
  const int variant = pick_variant(o ? o->variant : SLIM_VARIANT_AUTO, B, H, T, d, dtype);
  // the MFMA products count arrivals per (matrix, head, batch chunk)
  const int zb = (B + 15) / 16;
  const int nmat = slim_path ? 2 : 3;
  const bool fast = variant != SLIM_VARIANT_GENERIC && H * nmat * zb < CTRL_INTS / 2;
  const int k_layout = o ? o->k_layout : SLIM_K_ROWMAJOR;
  if (k_layout != SLIM_K_ROWMAJOR && k_layout != SLIM_K_BANDED) return SLIM_ERR_ARG;
  if (k_layout == SLIM_K_BANDED) {
    // decided before anything is appended: the decode step inside must be the stream kernel's
    if (!slim_path) return SLIM_ERR_ARG;
    DeviceState* dev = device_state();
    if (!fast || t_stride % 32 != 0 || !dev || !stream_kernel_fits(*dev, p.geom, rope != nullptr)) return SLIM_ERR_LAYOUT;
  }
  ProjArgs pa{};
  pa.Cpart = (const float*)c.x; pa.outpart = (float*)(ws + bb.off_dpart); pa.counters = (int*)(ws + p.off_ctrl);
  pa.seq_lens = lens; pa.B = B; pa.T = T; pa.H = H; pa.d_k = d_k; pa.rows = d; pa.e = d;
  pa.nsplit = 1; pa.mscale = 1.0f;

  StageTimer tm(o, st);
  if (fast) {
    // q, k (and v) in one launch; the new rows go straight into the caches
    launch_zero_ints(pa.counters, CTRL_INTS / 2, st);
    pa.nmat = nmat; pa.csw = dense_row_splits(H, nmat, d, d, B);
    pa.Wm[0] = (const uint16_t*)c.W_Q; pa.outm[0] = q; pa.role[0] = 1;
    pa.Wm[1] = (const uint16_t*)c.W_K; pa.outm[1] = nullptr; pa.role[1] = 2;
    pa.Wm[2] = (const uint16_t*)c.W_V; pa.outm[2] = nullptr; pa.role[2] = 3;
    pa.Kc = (uint16_t*)c.Kcache; pa.Vc = (uint16_t*)c.Vcache; pa.c_bstride = t_stride * d;
    pa.k_banded = k_layout == SLIM_K_BANDED;
    pa.rope = rope; pa.rotate_k = slim_path ? 0 : 1;
    launch_dense_mfma(pa, st);
  } else {
    launch_project(dtype, (const float*)c.x, c.W_Q, d, d, 1, d, q, B, st);      // one "head" as wide as the matrix
    launch_project(dtype, (const float*)c.x, c.W_K, d, d, 1, d, knew, B, st);
    if (!slim_path) launch_project(dtype, (const float*)c.x, c.W_V, d, d, 1, d, vnew, B, st);
    launch_append(dtype, knew, slim_path ? nullptr : vnew, c.Kcache, slim_path ? nullptr : c.Vcache,
                  t_stride * d, lens, T, d, d_k, rope, q, slim_path ? 0 : 1, B, st);
  }
  if (int rc = launch_status()) return rc;
  tm.mark();

  slim_opts inner = o ? *o : slim_opts{};
  inner.dtype = dtype;
  inner.workspace = ws;
  inner.workspace_bytes = p.total;
  inner.stage_ms = nullptr;
  int rc;
  if (slim_path) {
    rc = slim_decode(q, c.Kcache, c.W_second, attn, B, H, T, d, &inner);
  } else {
    inner.rope_table = nullptr;                       // the cache already holds the rotated keys
    rc = vanilla_kv_decode(q, c.Kcache, c.Vcache, attn, B, H, T, d, &inner);
  }
  if (rc) return rc;
  tm.mark();
  if (fast) {
    pa.Cpart = attn; pa.nmat = 1; pa.csw = dense_row_splits(H, 1, d, d, B);
    pa.Wm[0] = (const uint16_t*)c.W_O; pa.outm[0] = (float*)c.y; pa.role[0] = 0;
    launch_dense_mfma(pa, st);
  } else {
    launch_project(dtype, attn, c.W_O, d, d, 1, d, (float*)c.y, B, st);
  }
  tm.mark();
  tm.finish();
  return launch_status();
}

}  // namespace

extern "C" size_t slim_workspace_bytes_block(int B, int H, int T, int d, int dtype) {
  if (B < 1 || H < 1 || T < 1 || d < 1) return 0;
  (void)dtype;
  return block_layout(make_plan(B, H, T, d, d), B, H, d).total;
}

extern "C" int slim_attention_block(const void* x, const void* W_Q, const void* W_K, const void* W_KV,
                                    const void* W_O, void* Kcache, void* y, int B, int H, int T, int d,
                                    const slim_opts* o) {
  BlockCall c{x, W_Q, W_K, nullptr, W_KV, W_O, Kcache, nullptr, y};
  return attention_block(true, c, B, H, T, d, o);
}

extern "C" int vanilla_attention_block(const void* x, const void* W_Q, const void* W_K, const void* W_V,
                                       const void* W_O, void* Kcache, void* Vcache, void* y, int B, int H,
                                       int T, int d, const slim_opts* o) {
  BlockCall c{x, W_Q, W_K, W_V, nullptr, W_O, Kcache, Vcache, y};
  return attention_block(false, c, B, H, T, d, o);
}
