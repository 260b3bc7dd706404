// Calls the C ABI of libespo.so from a plain HIP host program (no Python, no PyTorch): reads a
// binary file of inputs, runs one espo_step, one espo_advantages, one espo_whiten on its result
// and one espo_advantages_packed (the [B, T] arrays taken as B full trajectories of T tokens
// stored back to back, terminal reward values[b]), then the pair with a workspace between them
// (espo_length_order, espo_advantages_ws, espo_whiten_from_ws), writes the outputs to another binary file.  The GPU test that drives it generates the inputs and compares the
// outputs with the CPU oracle.
//
// input file (little endian): int32 B, V, T; float tau; uint64 seed; int32 step; espo_params;
//   float logits[B*V]; float values[B]; float z[B]; uint8 alive[B]; int32 stop_step[B];
//   float rewards[B*T]; float vals2[B*T]; int32 lengths[B]; uint8 stopped[B]
// output file: int32 tokens[B]; float regret[B]; float z[B]; uint8 alive[B]; int32 stop_step[B];
//   float logprob[B]; float entropy[B]; float td[B*T]; float adv[B*T];
//   float whitened[B*T] (0 beyond the lengths); float td_packed[B*T]; float adv_packed[B*T];
//   int32 order[B]; float adv_ws[B*T]; float whitened_from_ws[B*T] (0 beyond the lengths)
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/espo.h"

#define CK(x)                                                                      \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } \
  } while (0)
#define EK(x)                                                                      \
  do {                                                                             \
    int r_ = (x);                                                                  \
    if (r_ != ESPO_OK) { std::fprintf(stderr, "%s: %s\n", #x, espo_strerror(r_)); return 3; } \
  } while (0)

template <typename T>
static bool rd(std::FILE* f, T* p, size_t n) { return std::fread(p, sizeof(T), n, f) == n; }
template <typename T>
static bool wr(std::FILE* f, const T* p, size_t n) { return std::fwrite(p, sizeof(T), n, f) == n; }

template <typename T>
static int to_device(T** d, const std::vector<T>& h) {
  CK(hipMalloc((void**)d, h.size() * sizeof(T) + 16));
  CK(hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
  return 0;
}

int main(int argc, char** argv) {
  if (argc != 3) { std::fprintf(stderr, "usage: abi_check <in> <out>\n"); return 1; }
  std::FILE* f = std::fopen(argv[1], "rb");
  if (!f) return 1;
  int32_t B, V, T, step;
  float tau;
  uint64_t seed;
  espo_params p;
  if (!rd(f, &B, 1) || !rd(f, &V, 1) || !rd(f, &T, 1) || !rd(f, &tau, 1) || !rd(f, &seed, 1) || !rd(f, &step, 1) ||
      !rd(f, &p, 1))
    return 1;
  std::vector<float> logits((size_t)B * V), values(B), z(B), rewards((size_t)B * T), vals2((size_t)B * T);
  std::vector<uint8_t> alive(B), stopped(B);
  std::vector<int32_t> stop_step(B), lengths(B);
  if (!rd(f, logits.data(), logits.size()) || !rd(f, values.data(), B) || !rd(f, z.data(), B) || !rd(f, alive.data(), B) ||
      !rd(f, stop_step.data(), B) || !rd(f, rewards.data(), rewards.size()) || !rd(f, vals2.data(), vals2.size()) ||
      !rd(f, lengths.data(), B) || !rd(f, stopped.data(), B))
    return 1;
  std::fclose(f);

  float *d_logits, *d_values, *d_z, *d_rewards, *d_vals2, *d_regret, *d_logprob, *d_entropy, *d_td, *d_adv;
  uint8_t *d_alive, *d_stopped;
  int32_t *d_stop_step, *d_lengths, *d_tokens;
  if (to_device(&d_logits, logits) || to_device(&d_values, values) || to_device(&d_z, z) || to_device(&d_alive, alive) ||
      to_device(&d_stop_step, stop_step) || to_device(&d_rewards, rewards) || to_device(&d_vals2, vals2) ||
      to_device(&d_lengths, lengths) || to_device(&d_stopped, stopped))
    return 2;
  CK(hipMalloc((void**)&d_tokens, B * 4));
  CK(hipMalloc((void**)&d_regret, B * 4));
  CK(hipMalloc((void**)&d_logprob, B * 4));
  CK(hipMalloc((void**)&d_entropy, B * 4));
  CK(hipMalloc((void**)&d_td, (size_t)B * T * 4));
  CK(hipMalloc((void**)&d_adv, (size_t)B * T * 4));
  float *d_wh, *d_tdp, *d_advp;
  void* d_ws;
  int64_t* d_cu;
  std::vector<int64_t> cu(B + 1);
  for (int b = 0; b <= B; ++b) cu[b] = (int64_t)b * T;
  if (to_device(&d_cu, cu)) return 2;
  CK(hipMalloc((void**)&d_wh, (size_t)B * T * 4));
  CK(hipMemset(d_wh, 0, (size_t)B * T * 4));
  CK(hipMalloc((void**)&d_tdp, (size_t)B * T * 4));
  CK(hipMalloc((void**)&d_advp, (size_t)B * T * 4));
  const size_t ws_bytes = espo_whiten_workspace_bytes(B, T);
  CK(hipMalloc(&d_ws, ws_bytes));
  // the workspace that lets espo_step split rows over workgroups: zero before its first use
  const size_t step_ws_bytes = espo_step_workspace_bytes(B, V, ESPO_F32);
  void* d_step_ws = nullptr;
  if (step_ws_bytes) {
    CK(hipMalloc(&d_step_ws, step_ws_bytes));
    CK(hipMemset(d_step_ws, 0, step_ws_bytes));
  }
  int32_t* d_order;
  float *d_adv2, *d_wh2;
  void* d_aws;
  const size_t aws_bytes = espo_advantages_ws_bytes(B);
  CK(hipMalloc((void**)&d_order, B * 4));
  CK(hipMalloc((void**)&d_adv2, (size_t)B * T * 4));
  CK(hipMalloc((void**)&d_wh2, (size_t)B * T * 4));
  CK(hipMemset(d_wh2, 0, (size_t)B * T * 4));
  CK(hipMalloc(&d_aws, aws_bytes));
  CK(hipMemset(d_aws, 0, aws_bytes));  // its first 256 bytes have to be zero before the first call
  hipStream_t stream;
  CK(hipStreamCreate(&stream));

  EK(espo_step(d_logits, ESPO_F32, B, V, V, tau, seed, step, d_values, &p, d_z, d_alive, d_stop_step, d_tokens, d_regret,
               d_logprob, d_entropy, d_step_ws, step_ws_bytes, stream));
  EK(espo_advantages(d_rewards, d_vals2, d_lengths, d_stopped, B, T, -1.0f, 1.0f, 0.95f, d_td, d_adv, stream));
  EK(espo_whiten(d_adv, d_lengths, B, T, 1e-8f, 1, 0, d_wh, nullptr, d_ws, ws_bytes, stream));
  EK(espo_advantages_packed(nullptr, d_values, d_vals2, d_cu, d_stopped, B, (int64_t)B * T, -1.0f, 1.0f, 0.95f, d_tdp,
                            d_advp, nullptr, stream));
  // the same advantages again, rows longest first, the rows' sums handed to the whitening (td is rewritten with the same bits)
  EK(espo_length_order(d_lengths, B, T, d_order, stream));
  EK(espo_advantages_ws(d_rewards, d_vals2, d_lengths, d_stopped, B, T, -1.0f, 1.0f, 0.95f, d_td, d_adv2, d_order, d_aws,
                        aws_bytes, stream));
  EK(espo_whiten_from_ws(d_adv2, d_lengths, B, T, 1e-8f, 1, 0, d_wh2, nullptr, d_aws, aws_bytes, stream));
  CK(hipStreamSynchronize(stream));

  std::vector<int32_t> tokens(B), order(B);
  std::vector<float> adv2((size_t)B * T), wh2((size_t)B * T);
  CK(hipMemcpy(order.data(), d_order, B * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(adv2.data(), d_adv2, adv2.size() * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(wh2.data(), d_wh2, wh2.size() * 4, hipMemcpyDeviceToHost));
  std::vector<float> regret(B), logprob(B), entropy(B), td((size_t)B * T), adv((size_t)B * T);
  std::vector<float> wh((size_t)B * T), tdp((size_t)B * T), advp((size_t)B * T);
  CK(hipMemcpy(tokens.data(), d_tokens, B * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(regret.data(), d_regret, B * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(z.data(), d_z, B * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(alive.data(), d_alive, B, hipMemcpyDeviceToHost));
  CK(hipMemcpy(stop_step.data(), d_stop_step, B * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(logprob.data(), d_logprob, B * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(entropy.data(), d_entropy, B * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(td.data(), d_td, td.size() * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(adv.data(), d_adv, adv.size() * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(wh.data(), d_wh, wh.size() * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(tdp.data(), d_tdp, tdp.size() * 4, hipMemcpyDeviceToHost));
  CK(hipMemcpy(advp.data(), d_advp, advp.size() * 4, hipMemcpyDeviceToHost));
  std::FILE* o = std::fopen(argv[2], "wb");
  if (!o) return 1;
  const bool ok = wr(o, tokens.data(), B) && wr(o, regret.data(), B) && wr(o, z.data(), B) && wr(o, alive.data(), B) &&
                  wr(o, stop_step.data(), B) && wr(o, logprob.data(), B) && wr(o, entropy.data(), B) &&
                  wr(o, td.data(), td.size()) &&
                  wr(o, adv.data(), adv.size()) && wr(o, wh.data(), wh.size()) && wr(o, tdp.data(), tdp.size()) &&
                  wr(o, advp.data(), advp.size()) && wr(o, order.data(), B) && wr(o, adv2.data(), adv2.size()) &&
                  wr(o, wh2.data(), wh2.size());
  std::fclose(o);
  std::printf("abi_check: version %d, B=%d V=%d T=%d, step workspace %zu bytes, done\n", espo_version(), B, V, T, step_ws_bytes);
  return ok ? 0 : 1;
}
