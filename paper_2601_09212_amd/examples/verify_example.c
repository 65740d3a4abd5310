/* A minimal C user of the library: no Python, no torch.  Generates seeded logits on the host,
 * uploads them, runs one cool_sd_verify call (Algorithm 1, verification stage, with the annealed
 * schedule of Eq. sdar) and prints the accepted length and next token of every sequence.
 *
 *   verify_example B L V seed [dump_file]
 *
 * With dump_file, inputs and outputs are also written there (int32 header {B, L, V, 1}, then
 * target f32 [B,L+1,V], draft f32 [B,L,V], tokens i32 [B,L], omega f32 [L], u_accept f32 [B,L],
 * u_resample f32 [B], accept_len i32 [B], next_token i32 [B], p_tok, q_tok, f f32 [B,L],
 * resid_mass f32 [B]) so that a test can check the call against an independent implementation.
 *
 * Build (what paper_2601_09212_amd/build.py does):
 *   hipcc -x c verify_example.c -I include -L paper_2601_09212_amd -lcool_sd -Wl,-rpath,'$ORIGIN/..' -o verify_example
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "cool_sd.h"

#define HIP_OK(call)                                                                      \
  do {                                                                                    \
    hipError_t e_ = (call);                                                               \
    if (e_ != hipSuccess) {                                                               \
      fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));                   \
      return 2;                                                                           \
    }                                                                                     \
  } while (0)

static uint64_t rng_state;
static uint32_t rng24(void) {                     /* 24 random bits */
  rng_state = rng_state * 6364136223846793005ULL + 1442695040888963407ULL;
  return (uint32_t)(rng_state >> 40);
}
static float rng_uniform(void) { return (float)rng24() * (1.0f / 16777216.0f); }
static float rng_normalish(void) {                /* sum of four uniforms, variance 1 */
  return (rng_uniform() + rng_uniform() + rng_uniform() + rng_uniform() - 2.0f) * 1.7320508f;
}

int main(int argc, char** argv) {
  if (argc < 5) {
    fprintf(stderr, "usage: %s B L V seed [dump_file]\n", argv[0]);
    return 1;
  }
  const int B = atoi(argv[1]), L = atoi(argv[2]), V = atoi(argv[3]);
  rng_state = (uint64_t)atoll(argv[4]) * 2654435761ULL + 12345ULL;
  if (B < 1 || L < 1 || V < 2) return 1;
  const size_t nt = (size_t)B * (L + 1) * V, nd = (size_t)B * L * V, nbl = (size_t)B * L;

  float* target = (float*)malloc(nt * sizeof(float));
  float* draft = (float*)malloc(nd * sizeof(float));
  int32_t* tokens = (int32_t*)malloc(nbl * sizeof(int32_t));
  float* omega = (float*)malloc((size_t)L * sizeof(float));
  float* u_acc = (float*)malloc(nbl * sizeof(float));
  float* u_res = (float*)malloc((size_t)B * sizeof(float));
  if (!target || !draft || !tokens || !omega || !u_acc || !u_res) return 2;
  for (size_t i = 0; i < nt; ++i) target[i] = 3.0f * rng_normalish();
  for (int b = 0; b < B; ++b)                       /* a draft that resembles the target */
    for (int i = 0; i < L; ++i)
      for (int x = 0; x < V; ++x)
        draft[((size_t)b * L + i) * V + x] = target[((size_t)b * (L + 1) + i) * V + x] + rng_normalish();
  for (size_t i = 0; i < nbl; ++i) {
    /* a plausible draft token: the best of eight random candidates under the draft's logits */
    const float* row = draft + i * V;
    int best = (int)(rng24() % (uint32_t)V);
    for (int c = 1; c < 8; ++c) {
      const int x = (int)(rng24() % (uint32_t)V);
      if (row[x] > row[best]) best = x;
    }
    tokens[i] = best;
    u_acc[i] = rng_uniform();
  }
  for (int b = 0; b < B; ++b) u_res[b] = rng_uniform();

  int rc = cool_sd_schedule(COOL_SD_SCHED_EXP, L, 1.1f, 0.7f, omega);
  if (rc != COOL_SD_OK) { fprintf(stderr, "cool_sd_schedule: %s\n", cool_sd_strerror(rc)); return 2; }

  cool_sd_params p;
  p.B = B; p.L = L; p.V = V; p.dtype = COOL_SD_F32;
  p.t_stride_b = (int64_t)(L + 1) * V; p.t_stride_l = V;
  p.d_stride_b = (int64_t)L * V; p.d_stride_l = V;
  p.omega_stride_b = 0;
  p.has_bonus = 1; p.top_k = 0; p.cfg_scale = 1.0f; p.temperature = 1.0f;
  p.resample_mode = COOL_SD_RESAMPLE_OPT; p.flags = 0;
  const size_t ws_bytes = cool_sd_workspace_bytes(&p);
  if (ws_bytes == 0) { fprintf(stderr, "invalid parameters\n"); return 2; }

  void *d_t, *d_d, *d_tok, *d_om, *d_ua, *d_ur, *d_tau, *d_next, *d_p, *d_q, *d_f, *d_R, *d_ws;
  HIP_OK(hipMalloc(&d_t, nt * 4)); HIP_OK(hipMalloc(&d_d, nd * 4)); HIP_OK(hipMalloc(&d_tok, nbl * 4));
  HIP_OK(hipMalloc(&d_om, (size_t)L * 4)); HIP_OK(hipMalloc(&d_ua, nbl * 4)); HIP_OK(hipMalloc(&d_ur, (size_t)B * 4));
  HIP_OK(hipMalloc(&d_tau, (size_t)B * 4)); HIP_OK(hipMalloc(&d_next, (size_t)B * 4));
  HIP_OK(hipMalloc(&d_p, nbl * 4)); HIP_OK(hipMalloc(&d_q, nbl * 4)); HIP_OK(hipMalloc(&d_f, nbl * 4));
  HIP_OK(hipMalloc(&d_R, (size_t)B * 4)); HIP_OK(hipMalloc(&d_ws, ws_bytes));
  HIP_OK(hipMemcpy(d_t, target, nt * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_d, draft, nd * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_tok, tokens, nbl * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_om, omega, (size_t)L * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_ua, u_acc, nbl * 4, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(d_ur, u_res, (size_t)B * 4, hipMemcpyHostToDevice));

  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));
  rc = cool_sd_workspace_init(d_ws, ws_bytes, stream);
  if (rc == COOL_SD_OK)
    rc = cool_sd_verify(&p, d_t, NULL, d_d, NULL, (const int32_t*)d_tok, (const float*)d_om, (const float*)d_ua,
                        (const float*)d_ur, (int32_t*)d_tau, (int32_t*)d_next, (float*)d_p, (float*)d_q, (float*)d_f,
                        (float*)d_R, d_ws, ws_bytes, stream);
  if (rc != COOL_SD_OK) { fprintf(stderr, "cool_sd_verify: %s\n", cool_sd_strerror(rc)); return 2; }
  HIP_OK(hipStreamSynchronize(stream));

  int32_t* tau = (int32_t*)malloc((size_t)B * 4);
  int32_t* next = (int32_t*)malloc((size_t)B * 4);
  float* pt = (float*)malloc(nbl * 4);
  float* qt = (float*)malloc(nbl * 4);
  float* f = (float*)malloc(nbl * 4);
  float* R = (float*)malloc((size_t)B * 4);
  if (!tau || !next || !pt || !qt || !f || !R) return 2;
  HIP_OK(hipMemcpy(tau, d_tau, (size_t)B * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(next, d_next, (size_t)B * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(pt, d_p, nbl * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(qt, d_q, nbl * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(f, d_f, nbl * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(R, d_R, (size_t)B * 4, hipMemcpyDeviceToHost));
  for (int b = 0; b < B; ++b)
    printf("sequence %d: accepted %d of %d draft tokens, next token %d (resampling mass %.6f)\n", b, tau[b], L,
           next[b], R[b]);

  if (argc > 5) {
    FILE* fp = fopen(argv[5], "wb");
    if (!fp) { perror(argv[5]); return 2; }
    const int32_t head[4] = {B, L, V, 1};
    int ok = fwrite(head, 4, 4, fp) == 4 && fwrite(target, 4, nt, fp) == nt && fwrite(draft, 4, nd, fp) == nd &&
             fwrite(tokens, 4, nbl, fp) == nbl && fwrite(omega, 4, (size_t)L, fp) == (size_t)L &&
             fwrite(u_acc, 4, nbl, fp) == nbl && fwrite(u_res, 4, (size_t)B, fp) == (size_t)B &&
             fwrite(tau, 4, (size_t)B, fp) == (size_t)B && fwrite(next, 4, (size_t)B, fp) == (size_t)B &&
             fwrite(pt, 4, nbl, fp) == nbl && fwrite(qt, 4, nbl, fp) == nbl && fwrite(f, 4, nbl, fp) == nbl &&
             fwrite(R, 4, (size_t)B, fp) == (size_t)B;
    if (fclose(fp) != 0 || !ok) { fprintf(stderr, "short write to %s\n", argv[5]); return 2; }
  }
  (void)hipStreamDestroy(stream);
  return 0;
}
