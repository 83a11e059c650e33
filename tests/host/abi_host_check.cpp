// Host-only exercise of the C ABI under AddressSanitizer / UBSan: argument validation and the planners.
#include <cstdio>
#include <cstdint>
#include <vector>
#include "qerl_nvfp4.h"
int main() {
  int bad = 0;
  void* fake = (void*)0x10000;
  // validation paths (never reach a launch)
  bad += nvfp4_quantize(nullptr, 4, 32, 32, (uint8_t*)fake, (uint8_t*)fake, nullptr, fake, 1 << 20, nullptr) != QERL_ERR_NULL;
  bad += nvfp4_lora_linear(fake, 2, 40, 40, (const uint8_t*)fake, (const uint8_t*)fake, (const float*)fake, 16, nullptr, nullptr, 0, 0.f, fake, 16, fake, 1 << 24, nullptr) != QERL_ERR_SHAPE;
  bad += qerl_workspace_status(nullptr, nullptr) != QERL_ERR_NULL;
  bad += qerl_status_from_error_word(5) != QERL_ERR_TIMEOUT;
  // planners over a grid of shapes
  long plans = 0;
  const int64_t Hs[] = {128, 512, 1040, 2048, 3584, 4096, 5120, 8192}, Is[] = {64, 640, 2368, 4096, 13824, 18944, 27648};
  for (int M = 1; M <= 16; ++M)
    for (int64_t H : Hs)
      for (int64_t I : Is)
        for (int64_t r : {0, 8, 16, 64}) {
          bad += aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(M, H, I, H, r, r, r) == 0;
          ++plans;
        }
  for (int M : {1, 8, 16, 17, 64, 128, 300, 4096})
    for (int64_t H : Hs) {
      const int64_t Ns[3] = {H, 1024, 1024}, rs[3] = {64, 64, 64};
      bad += aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(M, H, Ns, rs, 3) == 0;
      bad += nvfp4_lora_linear_workspace_bytes(M, 27648, H, 64) == 0;
      bad += nvfp4_lora_linear_swiglu_workspace_bytes(M, H, 27648, 64) == 0;
      bad += nvfp4_lora_linear_backward_workspace_bytes(M, 27648, H, 64) == 0;
      bad += mxfp4_lora_linear_native_workspace_bytes(M, 27648, H, 64) < mxfp4_linear_native_workspace_bytes(M, 27648, H);
      qerl_backward_desc bd[3] = {};
      for (int i = 0; i < 3; ++i) { bd[i].N = Ns[i]; bd[i].r = 64; }
      bad += nvfp4_lora_linear_backward_group_workspace_bytes(M, H, bd, 3) < nvfp4_lora_linear_backward_workspace_bytes(M, H, H, 64);
      plans += 6;
    }
  {
    // the new entry points' validation: descriptors on the host, nothing launched
    qerl_backward_desc bd[2] = {};
    for (auto& d : bd) { d.dy_bf16 = fake; d.lddy = 32; d.N = 32; d.packed_t = fake; d.tensor_scale = (const float*)fake; d.r = 0; }
    bad += nvfp4_lora_linear_backward_group(nullptr, 4, 64, 64, bd, 2, fake, 64, nullptr, 0, nullptr) != QERL_ERR_WORKSPACE;
    bd[1].N = 30;
    bad += nvfp4_lora_linear_backward_group(nullptr, 4, 64, 64, bd, 2, fake, 64, fake, 1 << 20, nullptr) != QERL_ERR_SHAPE;
    bad += nvfp4_lora_linear_backward_group(nullptr, 4, 64, 64, bd, 5, fake, 64, fake, 1 << 20, nullptr) != QERL_ERR_SHAPE;
    bad += mxfp4_lora_linear_native(fake, 4, 64, 64, fake, 8, fake, fake, 12, 1.f, nullptr, fake, 8, fake, 1 << 30, nullptr) != QERL_ERR_SHAPE;
    bad += mxfp4_lora_linear_native(fake, 4, 64, 64, fake, 8, nullptr, fake, 8, 1.f, nullptr, fake, 8, fake, 1 << 30, nullptr) != QERL_ERR_NULL;
    bad += mxfp4_lora_linear_native(fake, 4, 64, 64, fake, 8, nullptr, nullptr, 0, 0.f, nullptr, fake, 8, fake, 16, nullptr) != QERL_ERR_WORKSPACE;
  }
  bad += nvfp4_prepack_bytes(27648, 5120) != (size_t)864 * 40 * 2304;
  printf("host check: %ld sizing calls, %d unexpected results\n", plans, bad);
  return bad != 0;
}
