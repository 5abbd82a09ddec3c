// Host side of the C ABI: argument validation, threshold folding (merged gate of
// Sec. 3.2 of the channel-gating paper), layout of the caller's `packed` buffer,
// kernel-family choice and launch sequencing.  No device memory is allocated here.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <new>
#include <string>
#include <vector>

#include "cg_internal.h"

namespace {

thread_local std::string g_err = "";

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
}  // namespace

namespace cg {
// records the calling thread's error text for cg_last_error(); returns `code`
int set_error(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}
}  // namespace cg

namespace {

int elem_bytes(int dtype) {
  switch (dtype) {
    case CG_F32: return 4;
    case CG_BF16: return 2;
    case CG_I8: return 1;
    case CG_I32: return 4;
    default: return 0;
  }
}

constexpr int kTables = 8;  // per-channel tables of 4-byte entries at the start of `packed`

struct Layout {
  size_t table_stride;   // bytes per table
  size_t w_base_off, w_base_bytes;
  size_t w_cond_off, w_cond_bytes;
  size_t wpk_base_off, wpk_cond_off;
  size_t total;
};

}  // namespace

struct cg_conv {
  cg_conv_desc d;           // copy of the descriptor (host pointers are dead after create)
  int ho, wo, c_cond;
  int variant;              // resolved CG_VARIANT_*
  cg::Mfma3Plan plan3;
  cg::TilePlan plan4;
  Layout lay;
  std::vector<uint32_t> staging;  // host image of the tables; kept alive for the async copy
};

namespace {

// Pure checks; no HIP call.  Fills geometry on success.
int validate(const cg_conv_desc* d, int* ho, int* wo) {
  if (!d) return fail(CG_EINVAL, "descriptor is NULL");
  if (d->struct_size != sizeof(cg_conv_desc))
    return fail(CG_EINVAL, "struct_size %u does not match this library's %zu", d->struct_size, sizeof(cg_conv_desc));
  if (d->n_max <= 0 || d->h <= 0 || d->w <= 0 || d->c_in <= 0 || d->c_out <= 0)
    return fail(CG_EINVAL, "n_max, h, w, c_in, c_out must be positive");
  if (d->stride < 1 || d->pad < 0) return fail(CG_EINVAL, "stride must be >= 1 and pad >= 0");
  if (d->kh <= 0 || d->kw <= 0) return fail(CG_EINVAL, "kernel size must be positive");
  if (!((d->kh == 3 && d->kw == 3) || (d->kh == 1 && d->kw == 1)))
    return fail(CG_EUNSUPPORTED, "kernel size %dx%d: only 3x3 and 1x1 are supported", d->kh, d->kw);
  if (d->pad >= d->kh && d->pad > 0) return fail(CG_EINVAL, "pad %d must be smaller than the kernel size", d->pad);
  if (d->c_base <= 0 || d->c_base > d->c_in) return fail(CG_EINVAL, "c_base must lie in (0, c_in]");
  if (d->groups < 0) return fail(CG_EINVAL, "groups must be >= 0");
  if (d->groups > 1) {
    if ((long long)d->c_base * d->groups != d->c_in)
      return fail(CG_EINVAL, "channel grouping needs c_base * groups == c_in (%d * %d != %d)", d->c_base, d->groups,
                  d->c_in);
    if (d->c_out % d->groups) return fail(CG_EINVAL, "channel grouping needs groups to divide c_out");
  }
  if (d->shuffle != 0 && d->shuffle != 1) return fail(CG_EINVAL, "shuffle must be 0 or 1");
  if (d->shuffle && d->groups <= 1) return fail(CG_EINVAL, "shuffle needs channel grouping (groups > 1)");
  if (!(d->tau_c >= 0.0f) || std::isinf(d->tau_c)) return fail(CG_EINVAL, "tau_c must be finite and >= 0");
  if (d->tile_hint < 0 || d->tile_hint >= (1 << 12)) return fail(CG_EINVAL, "tile_hint has bits outside its three fields");
  if (d->in_dtype != CG_F32 && d->in_dtype != CG_BF16 && d->in_dtype != CG_I8)
    return fail(CG_EINVAL, "in_dtype must be CG_F32, CG_BF16 or CG_I8");
  if (d->in_dtype == CG_I8) {
    if (d->delta_hi) return fail(CG_EUNSUPPORTED, "the upper gate threshold (delta_hi) exists for float inputs only");
    if (d->out_dtype != CG_I32 && d->out_dtype != CG_I8)
      return fail(CG_EINVAL, "int8 inputs need out_dtype CG_I32 or CG_I8");
    if (d->rq_shift < 0 || d->rq_shift > 31) return fail(CG_EINVAL, "rq_shift must lie in [0, 31]");
  } else if (d->out_dtype != CG_F32 && d->out_dtype != CG_BF16) {
    return fail(CG_EINVAL, "float inputs need out_dtype CG_F32 or CG_BF16");
  }
  if (d->epilogue & ~(CG_EPI_RELU | CG_EPI_AFFINE | CG_EPI_RESIDUAL)) return fail(CG_EINVAL, "unknown epilogue flag");
  if (d->variant != CG_VARIANT_AUTO && d->variant != CG_VARIANT_NAIVE && d->variant != CG_VARIANT_MFMA_ROWS &&
      d->variant != CG_VARIANT_TILE)
    return fail(CG_EINVAL, "unknown variant %d", d->variant);
  if (d->x_pixel_stride != 0 && d->x_pixel_stride < d->c_in)
    return fail(CG_EINVAL, "x_pixel_stride must be 0 or >= c_in");
  const int span_h = d->h + 2 * d->pad - d->kh, span_w = d->w + 2 * d->pad - d->kw;
  if (span_h < 0 || span_w < 0) return fail(CG_EINVAL, "kernel larger than the padded input");
  *ho = span_h / d->stride + 1;
  *wo = span_w / d->stride + 1;
  const long long m = (long long)d->n_max * *ho * *wo;
  if (m * (long long)d->c_out >= (1ll << 40)) return fail(CG_EUNSUPPORTED, "output too large");
  if (!d->w_base) return fail(CG_EINVAL, "w_base is NULL");
  const bool gated = d->c_base < d->c_in;
  if (gated && !d->w_cond) return fail(CG_EINVAL, "w_cond is NULL for a gated layer");
  if (gated) {
    if (d->in_dtype == CG_I8) {
      if (!d->gate_thr_i32) return fail(CG_EINVAL, "gate_thr_i32 is NULL for a gated int8 layer");
    } else {
      if (!d->gate_mean || !d->gate_var || !d->delta)
        return fail(CG_EINVAL, "gate_mean, gate_var and delta are required for a gated float layer");
      if (std::isnan(d->gate_eps)) return fail(CG_EINVAL, "gate_eps is NaN");
      for (int c = 0; c < d->c_out; ++c) {
        if (std::isnan(d->gate_mean[c]) || std::isnan(d->gate_var[c]) || std::isnan(d->delta[c]) ||
            (d->delta_hi && std::isnan(d->delta_hi[c])))
          return fail(CG_EINVAL, "NaN in the gate statistics of channel %d", c);
        if (std::isinf(d->gate_mean[c]) || std::isinf(d->gate_var[c]))
          return fail(CG_EINVAL, "infinite gate statistics in channel %d", c);
        if ((double)d->gate_var[c] + (double)d->gate_eps < 0.0)
          return fail(CG_EINVAL, "gate_var + gate_eps is negative in channel %d", c);
      }
    }
  }
  return CG_OK;
}

Layout make_layout(const cg_conv_desc& d, size_t wpk_base_bytes, size_t wpk_cond_bytes) {
  Layout l{};
  const size_t eb = (size_t)elem_bytes(d.in_dtype);
  const size_t taps = (size_t)d.kh * d.kw;
  l.table_stride = align256((size_t)d.c_out * 4);
  size_t off = l.table_stride * kTables;
  l.w_base_bytes = (size_t)d.c_out * taps * d.c_base * eb;
  l.w_cond_bytes = (size_t)d.c_out * taps * (size_t)(d.c_in - d.c_base) * eb;
  l.w_base_off = off;
  off += align256(l.w_base_bytes);
  l.w_cond_off = off;
  off += align256(l.w_cond_bytes);
  l.wpk_base_off = off;
  off += align256(wpk_base_bytes);
  l.wpk_cond_off = off;
  off += align256(wpk_cond_bytes);
  l.total = off;
  return l;
}

struct Plans {
  cg::Mfma3Plan v3;
  cg::TilePlan v4;
  int variant;
  size_t wpk_base_bytes, wpk_cond_bytes;
};

// compute units of the current device (256 where no device answers: the plan is then the MI355X one)
int cu_count() {
  static int cached = 0;
  if (cached > 0) return cached;
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) {
    cached = n;
    return n;
  }
  (void)hipGetLastError();
  return 256;
}

int resolve_variant(const cg_conv_desc& d, Plans* pl) {
  pl->v4 = cg::tile_plan(d, cu_count());
  pl->v3 = cg::mfma3_plan(d, cu_count());
  if (d.variant == CG_VARIANT_TILE && !pl->v4.ok)
    return fail(CG_EUNSUPPORTED, "the large-tile matrix-core kernel does not cover this shape/dtype");
  if (d.variant == CG_VARIANT_MFMA_ROWS && !pl->v3.ok)
    return fail(CG_EUNSUPPORTED, "the row-tiled matrix-core kernel does not cover this shape/dtype");
  int v = d.variant;
  if (v == CG_VARIANT_AUTO) v = pl->v3.ok ? CG_VARIANT_MFMA_ROWS : pl->v4.ok ? CG_VARIANT_TILE : CG_VARIANT_NAIVE;
  pl->variant = v;
  pl->wpk_base_bytes = v == CG_VARIANT_TILE ? pl->v4.wpk_base_bytes : v == CG_VARIANT_MFMA_ROWS ? pl->v3.wpk_base_bytes : 0;
  pl->wpk_cond_bytes = v == CG_VARIANT_TILE ? pl->v4.wpk_cond_bytes : v == CG_VARIANT_MFMA_ROWS ? pl->v3.wpk_cond_bytes : 0;
  return CG_OK;
}

inline uint32_t f2u(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  return u;
}

}  // namespace

namespace {

// Scratch for cg_conv_forward_noalloc: what cg_conv_forward takes as its `workspace` argument (the
// batch's decision bitmap when only counts are asked for, and the first-pass counts and the channel
// mask of the channel-wise gate).  Every GPU the library runs on holds its own copy of the array
// until the process ends.  In host code the array's name is not a device address: the address is
// asked for once per device and kept.
constexpr size_t kScratchBytes = (size_t)16 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
void* g_scratch_ptr[kMaxDevices] = {};

// the current device's copy of `scratch` (NULL with the error text set on failure)
void* scratch_of_current_device() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fail(CG_EHIP, "no usable current device for the scratch array: %s", hipGetErrorString(e));
    return nullptr;
  }
  void* ptr = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (ptr) return ptr;
  e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !ptr) {
    fail(CG_EHIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
    return nullptr;
  }
  __atomic_store_n(&g_scratch_ptr[dev], ptr, __ATOMIC_RELEASE);   // (two threads may both ask: same answer)
  return ptr;
}

}  // namespace

extern "C" {

const char* cg_last_error(void) { return g_err.c_str(); }

size_t cg_conv_packed_bytes(const cg_conv_desc* desc) {
  int ho, wo;
  if (validate(desc, &ho, &wo) != CG_OK) return 0;
  Plans pl;
  if (resolve_variant(*desc, &pl) != CG_OK) return 0;
  return make_layout(*desc, pl.wpk_base_bytes, pl.wpk_cond_bytes).total;
}

int cg_conv_create(cg_conv** out, const cg_conv_desc* desc, void* hip_stream) {
  if (!out) return fail(CG_EINVAL, "out is NULL");
  *out = nullptr;
  int ho, wo;
  int rc = validate(desc, &ho, &wo);
  if (rc != CG_OK) return rc;
  const cg_conv_desc& d = *desc;
  Plans pl;
  rc = resolve_variant(d, &pl);
  if (rc != CG_OK) return rc;
  const int variant = pl.variant;
  const cg::Mfma3Plan& plan3 = pl.v3;
  const Layout lay = make_layout(d, pl.wpk_base_bytes, pl.wpk_cond_bytes);
  if (!d.packed) return fail(CG_EINVAL, "packed is NULL");
  if (((uintptr_t)d.packed & 255) != 0) return fail(CG_EINVAL, "packed must be 256-byte aligned");
  if (d.packed_bytes < lay.total)
    return fail(CG_EINVAL, "packed_bytes %zu is smaller than the %zu required", d.packed_bytes, lay.total);

  cg_conv* h = new (std::nothrow) cg_conv();
  if (!h) return fail(CG_ENOMEM, "out of host memory");
  h->d = d;
  if (h->d.x_pixel_stride == 0) h->d.x_pixel_stride = d.c_in;
  h->ho = ho;
  h->wo = wo;
  h->c_cond = d.c_in - d.c_base;
  h->variant = variant;
  h->plan3 = plan3;
  h->plan4 = pl.v4;
  h->lay = lay;

  // Host image of the per-channel tables.
  //   float path: 0 thr, 1 thr_hi, 2 sc0, 3 sh0, 4 sc1, 5 sh1
  //   int path:   0 thr, 2 mult0, 3 mult1, 4 bias
  const size_t tw = lay.table_stride / 4;
  try {
    h->staging.assign(tw * kTables, 0u);
  } catch (...) {
    delete h;
    return fail(CG_ENOMEM, "out of host memory");
  }
  uint32_t* t = h->staging.data();
  const bool gated = d.c_base < d.c_in;
  const float inf = std::numeric_limits<float>::infinity();
  for (int c = 0; c < d.c_out; ++c) {
    if (d.in_dtype == CG_I8) {
      t[0 * tw + c] = (uint32_t)(gated ? d.gate_thr_i32[c] : std::numeric_limits<int32_t>::min());
      t[2 * tw + c] = (uint32_t)(d.rq_mult0 ? d.rq_mult0[c] : 1);
      t[3 * tw + c] = (uint32_t)(d.rq_mult1 ? d.rq_mult1[c] : 1);
      t[4 * tw + c] = (uint32_t)(d.rq_bias ? d.rq_bias[c] : 0);
    } else {
      float lo = -inf, hi = inf;
      if (gated) {
        // merged gate: compare the raw partial sum with E + Delta*sqrt(Var+eps); never form inf*0
        const double sd = std::sqrt((double)d.gate_var[c] + (double)d.gate_eps);
        const double dl = d.delta[c];
        lo = std::isinf(dl) ? (dl < 0 ? -inf : inf) : (float)((double)d.gate_mean[c] + dl * sd);
        if (d.delta_hi) {
          const double dh = d.delta_hi[c];
          hi = std::isinf(dh) ? (dh < 0 ? -inf : inf) : (float)((double)d.gate_mean[c] + dh * sd);
        }
      }
      t[0 * tw + c] = f2u(lo);
      t[1 * tw + c] = f2u(hi);
      t[2 * tw + c] = f2u(d.scale0 ? d.scale0[c] : 1.0f);
      t[3 * tw + c] = f2u(d.shift0 ? d.shift0[c] : 0.0f);
      t[4 * tw + c] = f2u(d.scale1 ? d.scale1[c] : 1.0f);
      t[5 * tw + c] = f2u(d.shift1 ? d.shift1[c] : 0.0f);
    }
  }
  // host pointers must not be used after create
  h->d.gate_mean = h->d.gate_var = h->d.delta = h->d.delta_hi = nullptr;
  h->d.gate_thr_i32 = nullptr;
  h->d.scale0 = h->d.shift0 = h->d.scale1 = h->d.shift1 = nullptr;
  h->d.rq_mult0 = h->d.rq_mult1 = h->d.rq_bias = nullptr;

  hipStream_t s = (hipStream_t)hip_stream;
  char* pk = (char*)d.packed;
  hipError_t e = hipMemcpyAsync(pk, t, lay.table_stride * kTables, hipMemcpyHostToDevice, s);
  if (e == hipSuccess)
    e = hipMemcpyAsync(pk + lay.w_base_off, d.w_base, lay.w_base_bytes, hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess && lay.w_cond_bytes)
    e = hipMemcpyAsync(pk + lay.w_cond_off, d.w_cond, lay.w_cond_bytes, hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess && variant != CG_VARIANT_NAIVE) {
    cg::Params p{};
    p.c_in = d.c_in;
    p.c_out = d.c_out;
    p.c_base = d.c_base;
    p.c_cond = h->c_cond;
    p.kh = d.kh;
    p.kw = d.kw;
    p.in_dtype = d.in_dtype;
    p.groups = d.groups > 1 ? d.groups : 1;
    p.cpg = d.c_out / p.groups;
    p.w_base = pk + lay.w_base_off;
    p.w_cond = pk + lay.w_cond_off;
    if (variant == CG_VARIANT_TILE)
      e = cg::launch_tile_pack(pl.v4, p, pk + lay.wpk_base_off, pk + lay.wpk_cond_off, s);
    else
      e = cg::launch_mfma3_pack(plan3, p, pk + lay.wpk_base_off, pk + lay.wpk_cond_off, s);
  }
  if (e != hipSuccess) {
    const int code = fail(CG_EHIP, "cg_conv_create: %s", hipGetErrorString(e));
    delete h;
    return code;
  }
  h->d.w_base = h->d.w_cond = nullptr;
  // set-up is the place to ask for this device's scratch address, so that a later
  // cg_conv_forward_noalloc (possibly under graph capture) only reads it
  if (!scratch_of_current_device()) {
    const std::string keep = g_err;
    delete h;
    g_err = keep;
    return CG_EHIP;
  }
  *out = h;
  return CG_OK;
}

namespace {
// Workspace layout: [decision bitmap of the batch][per-(image, channel) counts of the first pass]
// [channel mask].  The row-tiled kernel counts fired gates from a decision bitmap; it goes to the
// workspace when the caller asks for counts without a bitmap, and so does the first pass of the
// channel-wise gate.  The other two areas exist only with the channel-wise gate.
struct WsLayout {
  size_t bitmap_off, bitmap_bytes, counts_off, counts_bytes, mask_off, mask_bytes, total;
};
WsLayout ws_layout(const cg_conv* h, int32_t n) {
  WsLayout w{};
  const size_t words = (size_t)(h->d.c_out + 31) / 32;
  const bool chan_gate = h->c_cond > 0 && h->d.tau_c > 0.0f;
  if ((h->variant == CG_VARIANT_MFMA_ROWS || h->variant == CG_VARIANT_TILE) && h->c_cond > 0)
    w.bitmap_bytes = align256((size_t)n * h->ho * h->wo * words * 4);
  if (chan_gate) {
    w.counts_bytes = align256((2 + (size_t)n * h->d.c_out) * 4);
    w.mask_bytes = align256((size_t)n * words * 4);
  }
  w.bitmap_off = 0;
  w.counts_off = w.bitmap_bytes;
  w.mask_off = w.counts_off + w.counts_bytes;
  w.total = w.mask_off + w.mask_bytes;
  return w;
}
}  // namespace

size_t cg_conv_workspace_bytes(const cg_conv* h, int32_t n) {
  if (!h || n <= 0) return 0;
  return ws_layout(h, n).total;
}

int cg_conv_info(const cg_conv* h, int32_t* ho, int32_t* wo) {
  if (!h) return -1;
  if (ho) *ho = h->ho;
  if (wo) *wo = h->wo;
  return h->variant;
}

}  // extern "C"

namespace {

int forward_impl(cg_conv* h, int32_t n, const void* x, const void* residual, void* y, uint32_t* bitmap,
                 uint32_t* counts, void* workspace, size_t workspace_bytes, void* hip_stream);

}  // namespace

extern "C" {

int cg_conv_forward(cg_conv* h, int32_t n, const void* x, const void* residual, void* y, uint32_t* bitmap,
                    uint32_t* counts, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return forward_impl(h, n, x, residual, y, bitmap, counts, workspace, workspace_bytes, hip_stream);
}

int cg_conv_forward_noalloc(cg_conv* h, int32_t n, const void* x, const void* residual, void* y, uint32_t* bitmap,
                            uint32_t* counts, void* hip_stream) {
  if (!h) return fail(CG_EINVAL, "handle is NULL");
  if (n < 0 || n > h->d.n_max) return fail(CG_EINVAL, "n = %d is outside [0, n_max = %d]", n, h->d.n_max);
  const size_t need = n > 0 ? cg_conv_workspace_bytes(h, n) : 0;
  if (need > kScratchBytes)
    return fail(CG_EUNSUPPORTED, "this call needs %zu bytes of scratch; the library's fixed scratch array holds %zu",
                need, kScratchBytes);
  void* ws = nullptr;
  if (need > 0) {
    ws = scratch_of_current_device();
    if (!ws) return CG_EHIP;
  }
  return forward_impl(h, n, x, residual, y, bitmap, counts, ws, need, hip_stream);
}

void cg_conv_destroy(cg_conv* h) { delete h; }

}  // extern "C"

namespace {

int forward_impl(cg_conv* h, int32_t n, const void* x, const void* residual, void* y, uint32_t* bitmap,
                 uint32_t* counts, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!h) return fail(CG_EINVAL, "handle is NULL");
  if (n < 0 || n > h->d.n_max) return fail(CG_EINVAL, "n = %d is outside [0, n_max = %d]", n, h->d.n_max);
  if (n == 0) return CG_OK;
  if (!x || !y) return fail(CG_EINVAL, "x and y must not be NULL");
  if ((h->d.epilogue & CG_EPI_RESIDUAL) && !residual)
    return fail(CG_EINVAL, "residual is NULL but the layer was created with CG_EPI_RESIDUAL");
  if (counts && ((uintptr_t)counts & 7)) return fail(CG_EINVAL, "counts must be 8-byte aligned");
  if (h->variant != CG_VARIANT_NAIVE &&
      ((((uintptr_t)x) | ((uintptr_t)y) | ((uintptr_t)residual) | ((uintptr_t)bitmap)) & 15))
    return fail(CG_EINVAL, "x, y, residual and bitmap must be 16-byte aligned");
  const size_t need = cg_conv_workspace_bytes(h, n);
  if (need > 0 && (!workspace || workspace_bytes < need))
    return fail(CG_EINVAL, "workspace of %zu bytes is smaller than the %zu required", workspace_bytes, need);
  if (need > 0 && ((uintptr_t)workspace & 255)) return fail(CG_EINVAL, "workspace must be 256-byte aligned");

  const cg_conv_desc& d = h->d;
  const char* pk = (const char*)d.packed;
  const Layout& l = h->lay;
  cg::Params p{};
  p.n = n;
  p.h = d.h;
  p.w = d.w;
  p.c_in = d.c_in;
  p.c_out = d.c_out;
  p.c_base = d.c_base;
  p.c_cond = h->c_cond;
  p.kh = d.kh;
  p.kw = d.kw;
  p.stride = d.stride;
  p.pad = d.pad;
  p.ho = h->ho;
  p.wo = h->wo;
  p.x_pixel_stride = d.x_pixel_stride;
  p.m_total = (long long)n * h->ho * h->wo;
  p.epilogue = d.epilogue;
  p.in_dtype = d.in_dtype;
  p.out_dtype = d.out_dtype;
  p.gated = h->c_cond > 0;
  p.rq_shift = d.rq_shift;
  p.rq_res_mult = d.rq_res_mult;
  p.words = (d.c_out + 31) / 32;
  p.groups = d.groups > 1 ? d.groups : 1;
  p.cpg = d.c_out / p.groups;
  p.shuffle = d.shuffle;
  const size_t ts = l.table_stride;
  p.thr_f = (const float*)(pk + 0 * ts);
  p.thr_hi_f = (const float*)(pk + 1 * ts);
  p.thr_i = (const int32_t*)(pk + 0 * ts);
  p.sc0 = (const float*)(pk + 2 * ts);
  p.sh0 = (const float*)(pk + 3 * ts);
  p.sc1 = (const float*)(pk + 4 * ts);
  p.sh1 = (const float*)(pk + 5 * ts);
  p.mult0 = (const int32_t*)(pk + 2 * ts);
  p.mult1 = (const int32_t*)(pk + 3 * ts);
  p.bias = (const int32_t*)(pk + 4 * ts);
  p.w_base = pk + l.w_base_off;
  p.w_cond = pk + l.w_cond_off;
  p.table_stride = ts;
  p.zeros = pk + 7 * ts;       // the last table is never written: zeros
  p.x = x;
  p.residual = residual;
  p.y = y;
  p.bitmap = bitmap;
  p.counts = counts;

  // The launch shape follows the batch of this call: a smaller batch than n_max is planned afresh
  // and the new plan is used if it reads the prepacked weights the same way.
  cg::Mfma3Plan plan3 = h->plan3;
  cg::TilePlan plan4 = h->plan4;
  if (n != d.n_max && h->variant != CG_VARIANT_NAIVE) {
    cg_conv_desc dn = d;
    dn.n_max = n;
    if (h->variant == CG_VARIANT_MFMA_ROWS) {
      const cg::Mfma3Plan q = cg::mfma3_plan(dn, cu_count());
      if (q.ok && q.cps == plan3.cps && q.grp_mode == plan3.grp_mode && q.gsp == plan3.gsp &&
          q.stages[0] == plan3.stages[0] && q.stages[1] == plan3.stages[1])
        plan3 = q;
    } else {
      const cg::TilePlan q = cg::tile_plan(dn, cu_count());
      if (q.ok && q.taps == plan4.taps && q.cps == plan4.cps && q.wn == plan4.wn && q.grp_mode == plan4.grp_mode &&
          q.gsp == plan4.gsp && q.stages[0] == plan4.stages[0] && q.stages[1] == plan4.stages[1])
        plan4 = q;
    }
  }

  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t e = hipSuccess;
  const WsLayout wl = ws_layout(h, n);
  char* ws = (char*)workspace;
  if (p.gated && d.tau_c > 0.0f) {
    // Channel-wise gate (Sec. 3.2): a first pass over the base path and the gate gives the fired
    // count of every (image, channel); the channels at or above tau_c * Ho * Wo form the mask that
    // the full pass ANDs into its decisions.
    const double need_d = std::ceil((double)d.tau_c * (double)((long long)h->ho * h->wo));
    const uint32_t need_u = need_d >= 4294967295.0 ? 0xffffffffu : (uint32_t)need_d;
    uint32_t* pre_counts = (uint32_t*)(ws + wl.counts_off);
    uint32_t* mask = (uint32_t*)(ws + wl.mask_off);
    cg::Params q = p;
    q.gate_only = 1;
    q.y = nullptr;
    q.counts = nullptr;
    q.bitmap = nullptr;
    if (h->variant == CG_VARIANT_MFMA_ROWS || h->variant == CG_VARIANT_TILE) {
      q.bitmap = (uint32_t*)(ws + wl.bitmap_off);
      e = h->variant == CG_VARIANT_TILE ? cg::launch_tile(plan4, q, pk + l.wpk_base_off, pk + l.wpk_cond_off, s)
                                        : cg::launch_mfma3(plan3, q, pk + l.wpk_base_off, pk + l.wpk_cond_off, s);
      if (e == hipSuccess) e = cg::launch_bitmap_chan_mask(q, q.bitmap, need_u, mask, s);
    } else {
      e = cg::launch_zero_u32(pre_counts, 2 + (size_t)n * d.c_out, s);
      q.counts = pre_counts;
      if (e == hipSuccess) e = cg::launch_naive(q, s);
      if (e == hipSuccess) e = cg::launch_chan_mask(pre_counts, n, d.c_out, p.words, need_u, mask, s);
    }
    p.chan_mask = mask;
  }
  if (e == hipSuccess && counts) e = cg::launch_zero_u32(counts, 2 + (size_t)n * d.c_out, s);
  if (e == hipSuccess && (h->variant == CG_VARIANT_MFMA_ROWS || h->variant == CG_VARIANT_TILE)) {
    const size_t bm_words = (size_t)p.m_total * p.words;
    if (!p.gated) {
      if (bitmap) e = cg::launch_zero_u32(bitmap, bm_words, s);   // a dense layer has no decisions
    } else if (counts && !bitmap) {
      p.bitmap = (uint32_t*)(ws + wl.bitmap_off);   // free again once the mask exists
    }
    if (e == hipSuccess)
      e = h->variant == CG_VARIANT_TILE ? cg::launch_tile(plan4, p, pk + l.wpk_base_off, pk + l.wpk_cond_off, s)
                                        : cg::launch_mfma3(plan3, p, pk + l.wpk_base_off, pk + l.wpk_cond_off, s);
    if (e == hipSuccess && counts && p.gated) e = cg::launch_bitmap_counts(p, p.bitmap, s);
  } else if (e == hipSuccess) {
    e = cg::launch_naive(p, s);
  }
  if (e != hipSuccess) return fail(CG_EHIP, "cg_conv_forward: %s", hipGetErrorString(e));
  return CG_OK;
}

}  // namespace
