// Host-side exercise of the C ABI for a build with -fsanitize=address,undefined (host code only;
// tests/test_abi_sanitized.py compiles the library's sources host-only together with this file and
// runs the result).  Every call here returns before anything is launched on a GPU: workspace
// planning, argument validation, error strings, the profiling bookkeeping with no recorded calls.
// What the sanitizers watch: the planners' size arithmetic at the edges of the supported range,
// reads of the dims / weights / layout structs, and the host-side bookkeeping arrays.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <initializer_list>
#include <vector>

#include "rom.h"

// The library's objects are compiled host-only here, so there is no device image to register: the
// registration hooks that the compiler's start-up code calls are satisfied by these no-ops (the
// test links them into the executable, ahead of the HIP runtime's), and the image symbols the
// objects refer to are defined as absolute zeros on the link line.  No kernel can be launched in
// this build, and nothing below tries to.
extern "C" {
void **__hipRegisterFatBinary(const void *) {
  static void *handle = nullptr;
  return &handle;
}
void __hipUnregisterFatBinary(void **) {}
void __hipRegisterFunction(void **, const void *, char *, const char *, unsigned, void *, void *, void *, void *, int *) {}
void __hipRegisterVar(void **, void *, char *, const char *, int, size_t, int, int) {}
void __hipRegisterManagedVar(void *, void **, void *, const char *, size_t, unsigned) {}
}

static int failures = 0;
#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) {                                                           \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      ++failures;                                                            \
    }                                                                        \
  } while (0)

static rom_dims dims_of(int d_model, int d_inner, int dt_rank, int E, int K, int Ex, int dtype, int gate_mode) {
  rom_dims d;
  d.d_model = d_model; d.d_inner = d_inner; d.d_state = 16; d.d_conv = 4; d.dt_rank = dt_rank;
  d.n_experts = E; d.top_k = K; d.n_experts_xdt = Ex; d.dtype = dtype; d.gate_mode = gate_mode;
  return d;
}

int main() {
  // an aligned host block standing in for "some non-NULL, 256-byte aligned pointer": never dereferenced
  // by the calls below (they fail validation, or have nothing to do, before any launch)
  std::vector<unsigned char> block(8192 + 256);
  unsigned char *addr = reinterpret_cast<unsigned char *>((reinterpret_cast<uintptr_t>(block.data()) + 255) / 256 * 256);
  rom_weights w_null;
  std::memset(&w_null, 0, sizeof(w_null));
  rom_weights w;
  w.w_router = addr; w.b_router = nullptr; w.w_in = addr; w.conv_w = reinterpret_cast<const float *>(addr);
  w.conv_b = nullptr; w.w_x = addr; w.w_dt = addr; w.dt_bias = reinterpret_cast<const float *>(addr);
  w.A_log = reinterpret_cast<const float *>(addr); w.D = reinterpret_cast<const float *>(addr); w.w_out = addr;

  // ---- planners over the paper's shapes and the edges of the supported range
  const rom_dims shapes[] = {
      dims_of(64, 128, 4, 4, 1, 4, ROM_DTYPE_F32, 0),        dims_of(1024, 2048, 64, 8, 1, 8, ROM_DTYPE_BF16, 0),
      dims_of(2048, 4096, 128, 8, 1, 8, ROM_DTYPE_BF16, 0),  dims_of(2048, 4096, 128, 16, 2, 16, ROM_DTYPE_BF16, 1),
      dims_of(2048, 4096, 128, 8, 1, 1, ROM_DTYPE_BF16, 0),  dims_of(8, 16, 1, 1, 1, 1, ROM_DTYPE_F32, 0),
      dims_of(4096, 8192, 256, 64, 8, 64, ROM_DTYPE_BF16, 1),
  };
  const int64_t batches[] = {1, 2, 7, 256, 65535};
  const int64_t lengths[] = {1, 3, 64, 4097, 16384, int64_t(1) << 20};
  for (const rom_dims &d : shapes) {
    for (int64_t B : batches)
      for (int64_t L : lengths) {
        if (B * L * d.top_k > (int64_t(1) << 30)) continue;
        const size_t bytes = rom_workspace_bytes(&d, B, L);
        CHECK(bytes > 0);
        rom_ws_layout lay;
        CHECK(rom_workspace_layout(&d, B, L, &lay) == ROM_OK);
        CHECK(lay.total_bytes == bytes);
        CHECK(lay.expert_idx < bytes && lay.logits < bytes && lay.xz < bytes && lay.g < bytes);
        CHECK(lay.xz % 256 == 0 && lay.g % 256 == 0);
        const size_t route = rom_route_workspace_bytes(&d, B * L);
        CHECK(route > 0 && route <= rom_workspace_bytes(&d, B * L, 1));
        if (B * L <= (int64_t(1) << 24)) {
          const size_t bwd = rom_backward_workspace_bytes(&d, B, L);
          CHECK(bwd > bytes);
        }
        const size_t ffn = rom_ffn_workspace_bytes(&d, 2 * d.d_model, B * L);
        CHECK(ffn > 0);
      }
  }
  // invalid or unsupported shapes: size 0 / an error code, never a plan
  {
    rom_dims d = shapes[0];
    rom_ws_layout lay;
    d.d_state = 8;   CHECK(rom_workspace_bytes(&d, 1, 8) == 0);  d = shapes[0];
    d.top_k = 5;     CHECK(rom_workspace_bytes(&d, 1, 8) == 0);  d = shapes[0];
    d.dtype = 7;     CHECK(rom_workspace_bytes(&d, 1, 8) == 0);  d = shapes[0];
    d.d_conv = 3;    CHECK(rom_workspace_layout(&d, 1, 8, &lay) == ROM_E_UNSUPPORTED);  d = shapes[0];
    d.top_k = 0;     CHECK(rom_workspace_layout(&d, 1, 8, &lay) == ROM_E_INVAL);  d = shapes[0];
    d.n_experts_xdt = 2;  CHECK(rom_workspace_layout(&d, 1, 8, &lay) == ROM_E_INVAL);  d = shapes[0];
    CHECK(rom_workspace_bytes(nullptr, 1, 8) == 0);
    CHECK(rom_workspace_layout(&d, 1, 8, nullptr) == ROM_E_INVAL);
    CHECK(rom_workspace_bytes(&d, -1, 8) == 0);
    CHECK(rom_backward_workspace_bytes(nullptr, 1, 8) == 0);
  }

  // ---- argument validation of the launching entry points: refused before any launch
  {
    const rom_dims d = shapes[0];
    CHECK(rom_layer_forward(&d, &w_null, nullptr, 1, 8, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == ROM_E_INVAL);
    CHECK(rom_layer_forward(nullptr, &w, addr, 1, 8, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_route(&d, &w_null, nullptr, 8, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == ROM_E_INVAL);
    CHECK(rom_step(&d, &w_null, nullptr, 4, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == ROM_E_INVAL);
    CHECK(rom_step_static(&d, &w_null, nullptr, 4, nullptr, nullptr, nullptr, nullptr) == ROM_E_INVAL);
    rom_grads g;
    std::memset(&g, 0, sizeof(g));
    CHECK(rom_layer_backward(&d, &w, addr, 1, 8, addr, addr + 4096, &g, addr, 4096, nullptr) == ROM_E_INVAL);   // NULL gradient pointers
    CHECK(rom_layer_backward(&d, &w, addr, 1, 8, addr, addr + 4096, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_layer_backward_saved(&d, &w, addr, 1, 8, addr, addr + 4096, &g, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_layer_backward_saved(&d, &w, addr, 0, 8, addr, addr + 4096, &g, addr, 4096, nullptr) == ROM_OK);
    {   // the block's backward: its own checks come before the layer's
      const float *nw = reinterpret_cast<const float *>(addr);
      float *dnw = reinterpret_cast<float *>(addr + 8192);
      CHECK(rom_block_backward_workspace_bytes(&d, 1, 8) > rom_backward_workspace_bytes(&d, 1, 8));
      CHECK(rom_block_backward_workspace_bytes(nullptr, 1, 8) == 0);
      CHECK(rom_block_backward(&d, &w, nullptr, 1e-5f, addr, 1, 8, addr, nullptr, addr + 4096, &g, dnw, addr, 4096, nullptr) == ROM_E_INVAL);
      CHECK(rom_block_backward(&d, &w, nw, -1.0f, addr, 1, 8, addr, nullptr, addr + 4096, &g, dnw, addr, 4096, nullptr) == ROM_E_INVAL);
      CHECK(rom_block_backward(&d, &w, nw, 1e-5f, addr, 1, 8, addr, nullptr, addr + 4096, &g, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
      CHECK(rom_block_backward(&d, &w, nw, 1e-5f, addr, 1, 8, addr, nullptr, addr, &g, dnw, addr, 4096, nullptr) == ROM_E_INVAL);        // d_x == x
      CHECK(rom_block_backward(&d, &w, nw, 1e-5f, addr, 1, 8, addr, nullptr, addr + 4096, &g, dnw, addr, 4096, nullptr) == ROM_E_WORKSPACE);
      CHECK(rom_block_backward(&d, &w, nw, 1e-5f, addr, 0, 8, addr, nullptr, addr + 4096, &g, dnw, addr, 4096, nullptr) == ROM_OK);
      CHECK(rom_block_backward_saved(&d, &w, nw, 1e-5f, addr, 1, 8, addr, nullptr, addr + 4096, &g, dnw, addr, 4096, nullptr) == ROM_E_WORKSPACE);
      CHECK(rom_block_backward_saved(&d, &w, nw, 1e-5f, addr, 1, 8, addr, nullptr, addr, &g, dnw, addr, 4096, nullptr) == ROM_E_INVAL);
      CHECK(rom_block_forward_train(&d, &w, nw, 1e-5f, addr, 1, 8, addr + 4096, addr, 4096, nullptr) == ROM_E_WORKSPACE);
      CHECK(rom_block_forward_train(&d, &w, nw, 1e-5f, addr, 1, 8, addr, addr, 4096, nullptr) == ROM_E_INVAL);          // out == x
      CHECK(rom_block_forward_train(&d, &w, nullptr, 1e-5f, addr, 1, 8, addr + 4096, addr, 4096, nullptr) == ROM_E_INVAL);
      CHECK(rom_block_forward_train(&d, &w, nw, 1e-5f, addr, 0, 8, addr + 4096, addr, 4096, nullptr) == ROM_OK);
    }
    // workspace too small
    CHECK(rom_layer_forward(&d, &w, addr, 1, 8, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 16, nullptr) == ROM_E_WORKSPACE);
    // sizes beyond the supported range
    const rom_dims d2 = shapes[3];
    CHECK(rom_layer_forward(&d2, &w, addr, 65536, 1, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_UNSUPPORTED);
    CHECK(rom_layer_forward(&d2, &w, addr, 1, (int64_t(1) << 29) + 1, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_UNSUPPORTED);
    CHECK(rom_layer_forward(&d2, &w, addr, 65535, 1, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_WORKSPACE);
    // empty input: a successful no-op
    CHECK(rom_layer_forward(&d, &w, addr, 0, 8, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_OK);
    CHECK(rom_layer_forward(&d, &w, addr, 2, 0, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_OK);
    CHECK(rom_step(&d, &w, addr, 0, nullptr, nullptr, addr + 4096, addr, 4096, nullptr) == ROM_OK);
    int32_t *ip = reinterpret_cast<int32_t *>(addr);
    float *fp = reinterpret_cast<float *>(addr);
    CHECK(rom_route(&d, &w, addr, 0, ip, fp, ip, ip, ip, ip, nullptr, addr, 4096, nullptr) == ROM_OK);
    // balance statistics: the mean over no tokens is undefined
    CHECK(rom_balance_stats(&d, fp, ip, 0, 1e-3f, fp, fp, fp, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_balance_stats(&d, nullptr, ip, 8, 1e-3f, fp, fp, fp, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_backward_workspace_bytes(&d2, 1, 64) > rom_workspace_bytes(&d2, 1, 64));
  }

  // ---- RoM on Mamba2: planning and validation
  {
    rom_mamba2_dims m;
    m.d_model = 2048; m.d_inner = 4096; m.d_state = 128; m.d_conv = 4; m.headdim = 64;
    m.n_experts = 8; m.top_k = 1; m.dtype = ROM_DTYPE_BF16; m.gate_mode = 0;
    for (int64_t B : {int64_t(1), int64_t(3), int64_t(4096)})
      for (int64_t L : {int64_t(1), int64_t(63), int64_t(16384), int64_t(1) << 17}) {
        if (B * L > (int64_t(1) << 24)) continue;
        const size_t bytes = rom_mamba2_workspace_bytes(&m, B, L);
        CHECK(bytes > 0);
        rom_mamba2_ws_layout lay;
        CHECK(rom_mamba2_workspace_layout(&m, B, L, &lay) == ROM_OK);
        CHECK(lay.total_bytes == bytes && lay.zxbcdt < bytes && lay.xbc < bytes && lay.yz < bytes && lay.g < bytes);
        CHECK(lay.zxbcdt % 256 == 0 && lay.g % 256 == 0);
      }
    rom_mamba2_dims bad = m;
    bad.d_state = 32;    CHECK(rom_mamba2_workspace_bytes(&bad, 1, 64) == 0);  bad = m;
    bad.headdim = 32;    CHECK(rom_mamba2_workspace_bytes(&bad, 1, 64) == 0);  bad = m;
    bad.dtype = ROM_DTYPE_F32;  CHECK(rom_mamba2_workspace_bytes(&bad, 1, 64) == 0);  bad = m;
    bad.d_inner = 4096 + 64;    CHECK(rom_mamba2_workspace_bytes(&bad, 1, 64) == 0);  bad = m;
    bad.top_k = 9;       CHECK(rom_mamba2_workspace_bytes(&bad, 1, 64) == 0);
    CHECK(rom_mamba2_workspace_bytes(nullptr, 1, 64) == 0);
    rom_mamba2_ws_layout lay;
    CHECK(rom_mamba2_workspace_layout(&m, 1, 64, nullptr) == ROM_E_INVAL);
    bad = m; bad.d_conv = 3;
    CHECK(rom_mamba2_workspace_layout(&bad, 1, 64, &lay) == ROM_E_UNSUPPORTED);
    rom_mamba2_weights mw;
    std::memset(&mw, 0, sizeof(mw));
    CHECK(rom_mamba2_forward(&m, &mw, addr, 1, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);   // NULL weights
    mw.w_router = addr; mw.w_in = addr; mw.conv_w = reinterpret_cast<const float *>(addr);
    mw.dt_bias = mw.A_log = mw.D = mw.norm_w = reinterpret_cast<const float *>(addr); mw.w_out = addr;
    CHECK(rom_mamba2_forward(&m, &mw, addr, 1, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_WORKSPACE);
    {
      float *st = reinterpret_cast<float *>(addr);
      CHECK(rom_mamba2_forward(&m, &mw, addr, 1, 64, 1e-5f, st, nullptr, addr + 4096, st, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);   // in-place state on a long sequence
      CHECK(rom_mamba2_step(&m, &mw, addr, 4, 1e-5f, nullptr, st, addr + 4096, addr, 4096, nullptr) == ROM_E_INVAL);
      CHECK(rom_mamba2_step(&m, &mw, addr, 4, 1e-5f, st, st, addr + 4096, addr, 4096, nullptr) == ROM_E_WORKSPACE);
      CHECK(rom_mamba2_step(&m, &mw, addr, 0, 1e-5f, nullptr, nullptr, addr + 4096, addr, 4096, nullptr) == ROM_OK);
    }
    CHECK(rom_mamba2_forward(&m, &mw, addr, 1, 64, -1.0f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_mamba2_forward(&m, &mw, addr, 0, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_OK);
    CHECK(rom_mamba2_forward(&m, &mw, addr, 1, 64, 1e-5f, nullptr, nullptr, addr, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);          // out == x
    CHECK(rom_mamba2_forward(nullptr, &mw, addr, 1, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
    {   // the pre-norm block: the layer's checks plus its own
      const float *nw = reinterpret_cast<const float *>(addr);
      CHECK(rom_mamba2_block_forward(&m, &mw, nullptr, 1e-5f, addr, 1, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
      CHECK(rom_mamba2_block_forward(&m, &mw, nw, -1.0f, addr, 1, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
      CHECK(rom_mamba2_block_forward(&m, &mw, nw, 1e-5f, addr, 1, 64, 1e-5f, nullptr, nullptr, addr, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
      CHECK(rom_mamba2_block_forward(&m, &mw, nw, 1e-5f, addr, 1, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_WORKSPACE);
      CHECK(rom_mamba2_block_forward(&m, &mw, nw, 1e-5f, addr, 0, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_OK);
      CHECK(rom_fold_norm_rows(7, addr, nw, addr, 4, 64, nullptr) == ROM_E_INVAL);
      CHECK(rom_fold_norm_rows(ROM_DTYPE_BF16, nullptr, nw, addr, 4, 64, nullptr) == ROM_E_INVAL);
      CHECK(rom_fold_norm_rows(ROM_DTYPE_BF16, addr, nw, addr, -1, 64, nullptr) == ROM_E_INVAL);
      CHECK(rom_fold_norm_rows(ROM_DTYPE_BF16, addr, nw, addr, 0, 64, nullptr) == ROM_OK);
    }
  }

  // ---- RoM on Gated DeltaNet: planning and validation
  {
    rom_gdn_dims m;
    m.d_model = 2048; m.n_heads = 32; m.d_k = 64; m.d_v = 64; m.d_conv = 4;
    m.n_experts = 8; m.top_k = 2; m.dtype = ROM_DTYPE_BF16; m.gate_mode = 1;
    for (int64_t B : {int64_t(1), int64_t(8), int64_t(4096)})
      for (int64_t L : {int64_t(1), int64_t(65), int64_t(2048), int64_t(1) << 17}) {
        if (B * L > (int64_t(1) << 23)) continue;
        const size_t bytes = rom_gdn_workspace_bytes(&m, B, L);
        CHECK(bytes > 0);
        rom_gdn_ws_layout lay;
        CHECK(rom_gdn_workspace_layout(&m, B, L, &lay) == ROM_OK);
        CHECK(lay.total_bytes == bytes && lay.proj < bytes && lay.qkv < bytes && lay.y < bytes);
        CHECK(lay.proj % 256 == 0 && lay.y % 256 == 0);
      }
    rom_gdn_dims bad = m;
    bad.d_k = 32;        CHECK(rom_gdn_workspace_bytes(&bad, 1, 64) == 0);  bad = m;
    bad.d_v = 128;       CHECK(rom_gdn_workspace_bytes(&bad, 1, 64) == 0);  bad = m;
    bad.n_heads = 6;     CHECK(rom_gdn_workspace_bytes(&bad, 1, 64) == 0);  bad = m;
    bad.dtype = ROM_DTYPE_F32;  CHECK(rom_gdn_workspace_bytes(&bad, 1, 64) == 0);
    CHECK(rom_gdn_workspace_bytes(nullptr, 1, 64) == 0);
    CHECK(rom_gdn_workspace_layout(&m, 1, 64, nullptr) == ROM_E_INVAL);
    rom_gdn_weights gw;
    std::memset(&gw, 0, sizeof(gw));
    CHECK(rom_gdn_forward(&m, &gw, addr, 1, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
    gw.w_router = addr; gw.w_in = addr; gw.conv_w = reinterpret_cast<const float *>(addr);
    gw.dt_bias = gw.A_log = gw.norm_w = reinterpret_cast<const float *>(addr); gw.w_out = addr;
    CHECK(rom_gdn_forward(&m, &gw, addr, 1, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_WORKSPACE);
    CHECK(rom_gdn_forward(&m, &gw, addr, 0, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_OK);
    float *st = reinterpret_cast<float *>(addr);
    CHECK(rom_gdn_forward(&m, &gw, addr, 1, 64, 1e-5f, nullptr, st, addr + 4096, nullptr, st, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_gdn_forward(&m, &gw, addr, 1, 64, 1e-5f, nullptr, nullptr, addr, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_gdn_step(&m, &gw, addr, 4, 1e-5f, nullptr, st, addr + 4096, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_gdn_step(&m, &gw, addr, 4, 1e-5f, st, st, addr + 4096, addr, 4096, nullptr) == ROM_E_WORKSPACE);
    CHECK(rom_gdn_step(&m, &gw, addr, 0, 1e-5f, nullptr, nullptr, addr + 4096, addr, 4096, nullptr) == ROM_OK);
    CHECK(rom_gdn_block_forward(&m, &gw, nullptr, 1e-5f, addr, 1, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_gdn_block_forward(&m, &gw, st, 1e-5f, addr, 1, 64, 1e-5f, nullptr, nullptr, addr, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_gdn_block_forward(&m, &gw, st, 1e-5f, addr, 1, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_E_WORKSPACE);
    CHECK(rom_gdn_block_forward(&m, &gw, st, 1e-5f, addr, 0, 64, 1e-5f, nullptr, nullptr, addr + 4096, nullptr, nullptr, addr, 4096, nullptr) == ROM_OK);
  }

  // ---- FFN-MoE layer, forward and backward: validation before any launch
  {
    const rom_dims d = shapes[0];
    rom_ffn_weights fw;
    fw.w_gate_up = addr; fw.w_down = addr;
    rom_ffn_grads fg;
    std::memset(&fg, 0, sizeof(fg));
    const int32_t *ip = reinterpret_cast<const int32_t *>(addr);
    const float *fp = reinterpret_cast<const float *>(addr);
    float *dg = reinterpret_cast<float *>(addr + 8192);
    const int32_t d_ff = 2 * d.d_model;
    CHECK(rom_ffn_backward_workspace_bytes(&d, d_ff, 64) > rom_ffn_workspace_bytes(&d, d_ff, 64));
    CHECK(rom_ffn_backward_workspace_bytes(&d, 24, 64) == 0);             // d_ff not a multiple of 16
    CHECK(rom_ffn_backward_workspace_bytes(nullptr, d_ff, 64) == 0);
    CHECK(rom_ffn_moe_forward(&d, d_ff, nullptr, 1, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr + 4096, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_ffn_moe_forward(&d, d_ff, &fw, 1, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr, addr, 4096, nullptr) == ROM_E_INVAL);       // out == x
    CHECK(rom_ffn_moe_forward(&d, d_ff, &fw, 1, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr + 4096, addr, 4096, nullptr) == ROM_E_WORKSPACE);
    CHECK(rom_ffn_moe_backward(&d, d_ff, &fw, fp, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr, addr + 4096, dg, &fg, addr, 4096, nullptr) == ROM_E_INVAL);   // NULL gradient pointers
    fg.d_w_gate_up = dg; fg.d_w_down = dg;
    CHECK(rom_ffn_moe_backward(&d, d_ff, &fw, fp, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr, addr + 4096, dg, &fg, addr, 4096, nullptr) == ROM_E_INVAL);   // pre-norm without d_norm_weight
    fg.d_norm_weight = dg;
    CHECK(rom_ffn_moe_backward(&d, d_ff, &fw, fp, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr, addr, dg, &fg, addr, 4096, nullptr) == ROM_E_INVAL);          // d_x == x
    CHECK(rom_ffn_moe_backward(&d, d_ff, &fw, fp, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr, addr + 4096, nullptr, &fg, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_ffn_moe_backward(&d, d_ff, &fw, fp, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr, addr + 4096, dg, &fg, addr, 4096, nullptr) == ROM_E_WORKSPACE);
    CHECK(rom_ffn_moe_backward(&d, d_ff, &fw, nullptr, 1e-5f, 0, addr, 0, ip, ip, ip, fp, addr, addr + 4096, dg, &fg, addr, 4096, nullptr) == ROM_OK);
    CHECK(rom_ffn_moe_backward_saved(&d, d_ff, &fw, fp, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr, addr + 4096, dg, &fg, addr, 4096, nullptr) == ROM_E_WORKSPACE);
    CHECK(rom_ffn_moe_backward_saved(&d, d_ff, &fw, fp, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr, addr, dg, &fg, addr, 4096, nullptr) == ROM_E_INVAL);
    CHECK(rom_ffn_moe_forward_train(&d, d_ff, &fw, fp, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr + 4096, addr, 4096, nullptr) == ROM_E_WORKSPACE);
    CHECK(rom_ffn_moe_forward_train(&d, d_ff, &fw, fp, 1e-5f, 1, addr, 8, ip, ip, ip, fp, addr, addr, 4096, nullptr) == ROM_E_INVAL);    // out == x
    CHECK(rom_ffn_moe_forward_train(&d, d_ff, &fw, fp, 1e-5f, 1, addr, 0, ip, ip, ip, fp, addr + 4096, addr, 4096, nullptr) == ROM_OK);
  }

  // ---- strings and the profiling bookkeeping
  CHECK(std::strcmp(rom_strerror(ROM_OK), "ok") == 0);
  for (int code : {ROM_E_INVAL, ROM_E_WORKSPACE, ROM_E_UNSUPPORTED, ROM_E_HIP, ROM_E_STATIC_LIMIT, -99})
    CHECK(std::strlen(rom_strerror(code)) > 5);
  for (int s = -1; s <= ROM_STAGE_COUNT; ++s) CHECK(rom_stage_name(s) != nullptr);
  CHECK(rom_profile_enable(0) == ROM_OK);
  CHECK(rom_profile_select(1u << ROM_STAGE_IN_PROJ) == ROM_OK);
  {
    double ms[ROM_STAGE_COUNT * 4];
    int n = -1;
    CHECK(rom_profile_collect(ms, &n) == ROM_OK && n == 0);
    CHECK(rom_profile_collect_calls(ms, 4, &n) == ROM_OK && n == 0);
    CHECK(rom_profile_collect(nullptr, &n) == ROM_E_INVAL);
  }
  CHECK(rom_profile_select(~0u) == ROM_OK);

  if (failures) {
    std::fprintf(stderr, "%d check(s) failed\n", failures);
    return 1;
  }
  std::printf("all checks passed\n");
  return 0;
}
