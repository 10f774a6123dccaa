/* A caller of the C ABI that uses nothing but the HIP runtime and tensorbleu.h: no PyTorch, no
 * C++.  It scores three candidates whose BLEU follows from the definitions in closed form and
 * prints one line per candidate: "<score> <expected>".
 *   0: candidate identical to its reference                  -> 1
 *   1: candidate = first 20 tokens of a 30-token reference   -> exp(1 - 30/20) (every p_n = 1)
 *   2: candidate shares no token with its reference          -> 0
 * Build (done by paper_2510_05485_amd/build.py):
 *   hipcc -x c c_caller.c -I include -L paper_2510_05485_amd -ltensorbleu -lamdhip64 -lm */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "tensorbleu.h"

#define CHECK(call)                                                          \
  do {                                                                       \
    hipError_t e_ = (call);                                                  \
    if (e_ != hipSuccess) {                                                  \
      fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));             \
      return 2;                                                              \
    }                                                                        \
  } while (0)

int main(void) {
  enum { B = 3, R = 1, L = 32 };
  int32_t cand[B][L], refs[B][R][L], cand_len[B] = {30, 20, 25}, ref_len[B][R] = {{30}, {30}, {28}};
  memset(cand, 0, sizeof cand);
  memset(refs, 0, sizeof refs);
  for (int p = 0; p < 30; ++p) {
    refs[0][0][p] = 100 + p;
    cand[0][p] = 100 + p;
    refs[1][0][p] = 200 + p;
    if (p < 20) cand[1][p] = 200 + p;
    if (p < 28) refs[2][0][p] = 300 + p;
    if (p < 25) cand[2][p] = 400 + p;
  }
  const double expected[B] = {1.0, exp(1.0 - 30.0 / 20.0), 0.0};

  tb_config_t cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.max_n = 4;                 /* weights all zero: uniform 1/N */
  cfg.smoothing = TB_SMOOTH_NONE;
  cfg.vocab_size = 1000;
  cfg.force_path = TB_PATH_AUTO;
  cfg.token_bytes = 4;

  const size_t ws_bytes = tensorbleu_workspace_bytes(B, R, L, L, &cfg);
  if (ws_bytes == 0) {
    fprintf(stderr, "unsupported shape\n");
    return 2;
  }
  void *d_cand, *d_refs, *d_cl, *d_rl, *d_ws, *d_out;
  CHECK(hipMalloc(&d_cand, sizeof cand));
  CHECK(hipMalloc(&d_refs, sizeof refs));
  CHECK(hipMalloc(&d_cl, sizeof cand_len));
  CHECK(hipMalloc(&d_rl, sizeof ref_len));
  CHECK(hipMalloc(&d_ws, ws_bytes));
  CHECK(hipMalloc(&d_out, B * sizeof(float)));
  CHECK(hipMemcpy(d_cand, cand, sizeof cand, hipMemcpyHostToDevice));
  CHECK(hipMemcpy(d_refs, refs, sizeof refs, hipMemcpyHostToDevice));
  CHECK(hipMemcpy(d_cl, cand_len, sizeof cand_len, hipMemcpyHostToDevice));
  CHECK(hipMemcpy(d_rl, ref_len, sizeof ref_len, hipMemcpyHostToDevice));

  int path_ok = 1;
  for (int path = TB_PATH_FUSED; path <= TB_PATH_GLOBAL; ++path) {
    cfg.force_path = path;
    const size_t need = tensorbleu_workspace_bytes(B, R, L, L, &cfg);
    void* ws = d_ws;
    if (need > ws_bytes) CHECK(hipMalloc(&ws, need));
    const int rc = tensorbleu_sentence(d_cand, L, (const int32_t*)d_cl, d_refs, L,
                                       (const int32_t*)d_rl, B, R, &cfg, (float*)d_out, NULL, ws,
                                       need, NULL);
    if (rc != TB_OK) {
      fprintf(stderr, "tensorbleu_sentence: %s\n", tensorbleu_status_string(rc));
      return 2;
    }
    CHECK(hipDeviceSynchronize());
    float out[B];
    CHECK(hipMemcpy(out, d_out, sizeof out, hipMemcpyDeviceToHost));
    for (int i = 0; i < B; ++i) {
      printf("%.7f %.7f\n", out[i], expected[i]);
      if (fabs(out[i] - expected[i]) > 1e-5) path_ok = 0;
    }
    if (ws != d_ws) CHECK(hipFree(ws));
  }
  hipFree(d_cand); hipFree(d_refs); hipFree(d_cl); hipFree(d_rl); hipFree(d_ws); hipFree(d_out);
  return path_ok ? 0 : 1;
}
