// Host <-> kernel interface of the Cool-SD library (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace csd {

// Everything a kernel needs, passed by value.  Pointers are device pointers.
struct KArgs {
  const void* t;            // target logits (conditional)
  const void* tu;           // target unconditional logits or nullptr
  const void* d;            // draft logits (nullptr: stand-alone resample from p)
  const void* du;           // draft unconditional logits or nullptr
  const int32_t* tokens;    // [B, L]
  const float* omega;       // [L] or [B, L]
  const float* u_acc;       // [B, L]
  const float* u_res;       // [B]
  int32_t* accept_len;      // [B]
  int32_t* next_token;      // [B]
  float* p_tok;             // [B, L] or nullptr
  float* q_tok;
  float* f;
  float* resid_mass;        // [B] or nullptr
  int64_t t_sb, t_sl, d_sb, d_sl, om_sb;   // element strides
  int32_t B, L, V, has_bonus, top_k, resample_mode, resample_only, aligned, nchunks;
  float cfg_scale, inv_T;
  // workspace
  uint32_t* seq_counter;    // [B]       rows of a sequence that have finished
  uint32_t* row_counter;    // [rows]    chunks of a row that have finished        (nchunks > 1)
  uint32_t* k2_counter;     // [B]       chunks of the resampled row that finished (nchunks > 1)
  uint32_t* hint;           // [B]       L - (earliest rejected position seen so far), 0 = none
  int32_t* acc;             // [B, L]    accept decisions
  int32_t* cand_tok;        // [B, L+1]  candidate draw of every row that may be sampled from
  float* cand_R;            // [B, L+1]  its mass
  float4* part;             // [rows, nchunks] partial (Ct, St, Cd, Sd)             (nchunks > 1)
  float4* rowstat;          // [rows]    combined (Ct, St, Cd, Sd)                  (nchunks > 1)
  float* chunk_R;           // [B, nchunks] residual mass per chunk                 (nchunks > 1)
};

// Enqueue the kernels of one verify (or stand-alone resample) call.  xf: the logit transform
// (guidance / temperature / top-k) is active.  Returns hipSuccess or the launch error.
hipError_t launch_verify(const KArgs& a, int dtype, bool xf, hipStream_t stream);

// Zero n 32-bit words.
hipError_t launch_zero(uint32_t* p, size_t n, hipStream_t stream);

}  // namespace csd
