// Sanitizer driver for the host side of the C ABI: the translation unit that validates
// descriptors and lays out the caller's buffers (csrc/cg_conv_api.hip) is compiled with
// -fsanitize=address,undefined on the host pass and linked into this program (the kernels come
// from the already built libcg_conv.so).  Everything called here returns before the first HIP
// call, so it runs on a host without a GPU.  Run by tests/test_sanitizers_cpu.py.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <limits>
#include <vector>

#include "cg_conv.h"

static int failures = 0;
#define EXPECT(c) do { if (!(c)) { std::printf("FAILED line %d: %s  [%s]\n", __LINE__, #c, cg_last_error()); ++failures; } } while (0)

struct Desc {
  cg_conv_desc d;
  std::vector<float> mean, var, delta;      // exactly c_out entries: a read past them is reported
  std::vector<int32_t> thr;
  explicit Desc(int c_out = 64) : mean(c_out, 0.f), var(c_out, 1.f), delta(c_out, 0.5f), thr(c_out, 0) {
    std::memset(&d, 0, sizeof d);
    d.struct_size = sizeof d;
    d.n_max = 2; d.h = 14; d.w = 14; d.c_in = 64; d.c_out = c_out; d.kh = d.kw = 3; d.stride = 1; d.pad = 1;
    d.c_base = 16; d.in_dtype = CG_BF16; d.out_dtype = CG_F32; d.epilogue = CG_EPI_RELU;
    d.w_base = (const void*)0x1000; d.w_cond = (const void*)0x2000;     // never dereferenced by validation
    d.gate_mean = mean.data(); d.gate_var = var.data(); d.delta = delta.data(); d.gate_thr_i32 = thr.data();
  }
};

static int create_code(cg_conv_desc& d) {
  cg_conv* h = nullptr;
  const int rc = cg_conv_create(&h, &d, nullptr);
  EXPECT(h == nullptr || rc == CG_OK);
  if (h) cg_conv_destroy(h);
  return rc;
}

int main() {
  { Desc a; EXPECT(cg_conv_packed_bytes(&a.d) >= 64u * 9 * 64 * 2); }
  { Desc a; a.d.in_dtype = CG_I8; a.d.out_dtype = CG_I8; EXPECT(cg_conv_packed_bytes(&a.d) > 0); }
  { Desc a; a.d.in_dtype = CG_F32; EXPECT(cg_conv_packed_bytes(&a.d) > 0); }                    // plain kernel
  { Desc a(40); EXPECT(cg_conv_packed_bytes(&a.d) > 0); }                                       // c_out not a multiple of 64
  { Desc a; a.d.kh = a.d.kw = 1; a.d.pad = 0; EXPECT(cg_conv_packed_bytes(&a.d) > 0); }
  { Desc a; a.d.kh = a.d.kw = 1; a.d.pad = 0; a.d.h = a.d.w = 1; a.d.n_max = 130; EXPECT(cg_conv_packed_bytes(&a.d) > 0); }
  { Desc a; a.d.groups = 4; a.d.shuffle = 1; EXPECT(cg_conv_packed_bytes(&a.d) > 0); }
  { Desc a; a.d.c_base = 8; a.d.variant = CG_VARIANT_TILE; EXPECT(cg_conv_packed_bytes(&a.d) > 0); }
  { Desc a; a.d.h = 3; a.d.w = 3; a.d.pad = 0; EXPECT(cg_conv_packed_bytes(&a.d) > 0); }        // one output pixel
  { Desc a; a.d.tile_hint = 2 | (1 << 4); a.d.variant = CG_VARIANT_TILE; EXPECT(cg_conv_packed_bytes(&a.d) > 0); }
  // rejections: every one must leave an error text and no handle
  EXPECT(cg_conv_packed_bytes(nullptr) == 0);
  { Desc a; a.d.struct_size = 8; EXPECT(cg_conv_packed_bytes(&a.d) == 0 && create_code(a.d) == CG_EINVAL); }
  { Desc a; a.d.n_max = 0; EXPECT(create_code(a.d) == CG_EINVAL); }
  { Desc a; a.d.c_base = 0; EXPECT(create_code(a.d) == CG_EINVAL); }
  { Desc a; a.d.c_base = 65; EXPECT(create_code(a.d) == CG_EINVAL); }
  { Desc a; a.d.kh = a.d.kw = 5; EXPECT(create_code(a.d) == CG_EUNSUPPORTED); }
  { Desc a; a.d.variant = 2; EXPECT(create_code(a.d) == CG_EINVAL); }
  { Desc a; a.d.variant = CG_VARIANT_MFMA_ROWS; a.d.in_dtype = CG_F32; EXPECT(create_code(a.d) == CG_EUNSUPPORTED); }
  { Desc a; a.d.groups = 3; EXPECT(create_code(a.d) == CG_EINVAL); }
  { Desc a; a.d.shuffle = 1; EXPECT(create_code(a.d) == CG_EINVAL); }
  { Desc a; a.d.tau_c = -1.f; EXPECT(create_code(a.d) == CG_EINVAL); }
  { Desc a; a.d.tile_hint = 1 << 12; EXPECT(create_code(a.d) == CG_EINVAL); }
  { Desc a; a.d.tile_hint = 4 | (2 << 4); a.d.variant = CG_VARIANT_TILE; EXPECT(create_code(a.d) == CG_EUNSUPPORTED); }   // c_out = 64
  { Desc a; a.delta[63] = std::numeric_limits<float>::quiet_NaN(); EXPECT(create_code(a.d) == CG_EINVAL); }
  { Desc a; a.var[0] = -1.f; EXPECT(create_code(a.d) == CG_EINVAL); }
  { Desc a; a.d.gate_mean = nullptr; EXPECT(create_code(a.d) == CG_EINVAL); }
  { Desc a; a.d.in_dtype = CG_I8; a.d.out_dtype = CG_I8; a.d.delta_hi = a.delta.data(); EXPECT(create_code(a.d) == CG_EUNSUPPORTED); }
  { Desc a; a.d.packed = nullptr; EXPECT(create_code(a.d) == CG_EINVAL); }                      // valid otherwise
  { Desc a; a.d.packed = (void*)0x10001; a.d.packed_bytes = 1u << 30; EXPECT(create_code(a.d) == CG_EINVAL); }  // misaligned
  { Desc a; a.d.packed = (void*)0x10000; a.d.packed_bytes = 16; EXPECT(create_code(a.d) == CG_EINVAL); }        // too small
  EXPECT(cg_conv_workspace_bytes(nullptr, 4) == 0);
  EXPECT(cg_conv_forward(nullptr, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == CG_EINVAL);
  EXPECT(cg_conv_forward_noalloc(nullptr, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == CG_EINVAL);
  EXPECT(cg_conv_info(nullptr, nullptr, nullptr) == -1);
  cg_conv_destroy(nullptr);
  EXPECT(cg_small_cin_conv(nullptr, nullptr, nullptr, nullptr, nullptr, 1, 8, 8, 3, 64, 7, 2, 3, 1, nullptr) == CG_EINVAL);
  EXPECT(cg_avgpool_fc(nullptr, nullptr, nullptr, nullptr, 1, 49, 512, 1000, nullptr) == CG_EINVAL);
  if (failures) { std::printf("%d checks failed\n", failures); return 1; }
  std::printf("abi sanitizer driver: ok\n");
  return 0;
}
