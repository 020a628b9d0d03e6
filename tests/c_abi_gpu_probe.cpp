// A caller of the library that uses nothing but the HIP runtime and include/qcache.h: no Python, no
// tensor library.  It runs a small bf16 stack (prefill of two prompts through three layers, then two
// decode steps) on inputs from a counter-based generator and writes every layer call's output, as raw
// bf16, to the file named on the command line; tests/test_gpu_native_caller.py regenerates the inputs,
// runs the oracle and compares.  Built by the package's build step (hipcc, host code only).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "qcache.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s (line %d)\n", #x, hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define QC_DO(x) do { qc_status s_ = (x); if (s_ != QC_OK) { std::fprintf(stderr, "%s: %s: %s (line %d)\n", #x, qc_status_str(s_), qc_last_error(), __LINE__); return 3; } } while (0)

// Element i of stream `tag`: a multiple of 1/32 in [-2, 2], exactly representable in bf16.  The same
// generator is written out in workloads/counter_inputs.py.
static inline float counter_value(uint32_t tag, uint32_t i) {
  uint32_t u = i * 2654435761u + tag * 40503u + 12345u;
  u ^= u >> 15;
  u *= 2246822519u;
  u ^= u >> 13;
  return ((int)(u % 129u) - 64) / 32.0f;
}
static inline uint16_t bf16_bits(float x) {   // exact for the generator's values (low 16 bits are zero)
  uint32_t b;
  std::memcpy(&b, &x, 4);
  return (uint16_t)(b >> 16);
}
static void fill(std::vector<uint16_t>& dst, uint32_t tag) {
  for (size_t i = 0; i < dst.size(); ++i) dst[i] = bf16_bits(counter_value(tag, (uint32_t)i));
}

int main(int argc, char** argv) {
  if (argc != 2) { std::fprintf(stderr, "usage: %s <output file>\n", argv[0]); return 1; }
  enum { N = 3, H = 2, D = 128, B = 2, STEPS = 2 };
  const uint8_t mask[N] = {0, 1, 0};
  const int32_t lens[B] = {150, 70}, vis_start[B] = {20, 0}, vis_len[B] = {100, 33};
  const int32_t cu[B + 1] = {0, lens[0], lens[0] + lens[1]};
  const int tokens = cu[B];

  qc_config cfg;
  std::memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = N; cfg.n_heads = H; cfg.head_dim = D; cfg.dtype = QC_BF16;
  cfg.max_batch = B; cfg.max_seq = 160; cfg.max_vis = 100; cfg.max_text = 80;
  cfg.lazy_mask = mask;
  const size_t kv_bytes = qc_kv_arena_bytes(&cfg), q_bytes = qc_q_arena_bytes(&cfg), ws_bytes = qc_decode_workspace_bytes(&cfg);
  if (!kv_bytes || !q_bytes || !ws_bytes) { std::fprintf(stderr, "configuration refused: %s\n", qc_last_error()); return 3; }

  void *kv_arena, *q_arena, *ws, *dq, *dk, *dv, *dout;
  const size_t prompt_bytes = (size_t)tokens * H * D * 2, step_bytes = (size_t)B * H * D * 2;
  HIP_OK(hipMalloc(&kv_arena, kv_bytes)); HIP_OK(hipMalloc(&q_arena, q_bytes)); HIP_OK(hipMalloc(&ws, ws_bytes));
  HIP_OK(hipMalloc(&dq, prompt_bytes)); HIP_OK(hipMalloc(&dk, prompt_bytes)); HIP_OK(hipMalloc(&dv, prompt_bytes)); HIP_OK(hipMalloc(&dout, prompt_bytes));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));

  qc_kvcache* kv = nullptr;
  qc_qcache* qc = nullptr;
  QC_DO(qc_kvcache_create(&cfg, kv_arena, kv_bytes, &kv));
  QC_DO(qc_qcache_create(&cfg, q_arena, q_bytes, &qc));
  QC_DO(qc_reset(kv, qc, B, vis_start, vis_len, 1, stream));

  std::FILE* f = std::fopen(argv[1], "wb");
  if (!f) { std::perror(argv[1]); return 1; }
  std::vector<uint16_t> hq((size_t)tokens * H * D), hk(hq.size()), hv(hq.size()), ho(hq.size());
  for (int l = 0; l < N; ++l) {   // prefill: tensors [token][head][dim], streams 3*l, 3*l+1, 3*l+2
    fill(hq, 3 * l); fill(hk, 3 * l + 1); fill(hv, 3 * l + 2);
    HIP_OK(hipMemcpyAsync(dq, hq.data(), prompt_bytes, hipMemcpyHostToDevice, stream));
    HIP_OK(hipMemcpyAsync(dk, hk.data(), prompt_bytes, hipMemcpyHostToDevice, stream));
    HIP_OK(hipMemcpyAsync(dv, hv.data(), prompt_bytes, hipMemcpyHostToDevice, stream));
    QC_DO(qc_prefill(kv, qc, l, mask[l], dq, dk, dv, dout, cu, (int64_t)H * D, D, vis_start, vis_len, 0.0f, stream));
    HIP_OK(hipMemcpyAsync(ho.data(), dout, prompt_bytes, hipMemcpyDeviceToHost, stream));
    HIP_OK(hipStreamSynchronize(stream));
    std::fwrite(ho.data(), 1, prompt_bytes, f);
  }
  std::vector<uint16_t> sq((size_t)B * H * D), sk(sq.size()), sv(sq.size()), so(sq.size());
  for (int t = 0; t < STEPS; ++t)
    for (int l = 0; l < N; ++l) {   // decode: tensors [sequence][head][dim], streams 100 + 3*(t*N + l) ...
      const uint32_t tag = 100 + 3 * (t * N + l);
      fill(sq, tag); fill(sk, tag + 1); fill(sv, tag + 2);
      HIP_OK(hipMemcpyAsync(dq, sq.data(), step_bytes, hipMemcpyHostToDevice, stream));
      HIP_OK(hipMemcpyAsync(dk, sk.data(), step_bytes, hipMemcpyHostToDevice, stream));
      HIP_OK(hipMemcpyAsync(dv, sv.data(), step_bytes, hipMemcpyHostToDevice, stream));
      QC_DO(qc_decode(kv, qc, l, mask[l], dq, dk, dv, dout, vis_start, vis_len, 0.0f, ws, ws_bytes, stream));
      HIP_OK(hipMemcpyAsync(so.data(), dout, step_bytes, hipMemcpyDeviceToHost, stream));
      HIP_OK(hipStreamSynchronize(stream));
      std::fwrite(so.data(), 1, step_bytes, f);
    }
  std::fclose(f);

  qc_stats_t st;
  QC_DO(qc_stats(kv, qc, &st));
  std::printf("k_bytes %lld\nv_bytes %lld\nq_bytes %lld\ntokens %lld\n", (long long)st.k_bytes, (long long)st.v_bytes, (long long)st.q_bytes, (long long)st.tokens);
  qc_kvcache_destroy(kv);
  qc_qcache_destroy(qc);
  HIP_OK(hipStreamDestroy(stream));
  HIP_OK(hipFree(kv_arena)); HIP_OK(hipFree(q_arena)); HIP_OK(hipFree(ws));
  HIP_OK(hipFree(dq)); HIP_OK(hipFree(dk)); HIP_OK(hipFree(dv)); HIP_OK(hipFree(dout));
  return 0;
}
