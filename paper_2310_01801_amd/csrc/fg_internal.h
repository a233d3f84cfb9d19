// Host-side plumbing shared by the translation units of the FastGen HIP library:
// the context, the workspace carve-up and the kernel launchers. Not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/fastgen.h"

// ---------------------------------------------------------------- workspace layout
// Every region starts on a 256-byte boundary. Offsets are in bytes from the workspace base.
struct fg_layout {
  // profiling scratch
  size_t rowstat;   // [U * G, n] float2  per query row (m, 1/l): softmax row = 2^(c q.k - m) / l, with m a
                    //                    shift at or near the row's largest scaled logit (log2 domain)
  size_t colsum;    // [U, n] double  cumulative attention score of every prompt token
  size_t bandcol;   // [U, n] double  the part of colsum inside the local band
  size_t keep;      // [U, n] uint8   0 = dropped, else 4 | class bits of the kept token
  size_t slot;      // [U, n] int32   exclusive prefix sum of keep (slot in the cache)
  // per-unit results and cache bookkeeping
  size_t policy;    // [U] int32
  size_t recov;     // [U, 5] double
  size_t kcount;    // [U, 5] int32
  size_t cap;       // [U] int32      slots reserved for the unit
  size_t off;       // [U + 1] int64  first slot of each unit in the pool
  size_t len;       // [U] int32      tokens held
  size_t flags;     // [8] int32      [0] pool overflow, [1] decode steps done
  // ragged cache pool (pool_tokens slots)
  size_t ck;        // [pool, d] dtype
  size_t cv;        // [pool, d] dtype
  size_t cscore;    // [pool] double
  size_t cpos;      // [pool] int32
  size_t ccls;      // [pool] uint8
  size_t clogit;    // [pool, G] double  this step's scaled logit of every held token, per query head (written
                    //                   for the units whose cumulative scores are kept)
  // decode scratch
  size_t chunk_off; // [U + 1] int32  first chunk of each unit in the flat work list
  size_t item_unit; // [max_chunks, 8] int32  work-item records: unit, chunk, cap, tokens held, pool offset lo/hi, policy word, 0
  size_t part;      // [max_chunks, G, d + 2] float  split-KV partial (max, sum, o) per query head
  size_t total;
  int64_t pool_tokens;
  int64_t max_chunks;
  int chunk;        // tokens per decode work item (128 or 256)
};

struct fastgen_ctx {
  fg_config cfg;
  fg_layout lay;
  char* ws;
  float scale;
  int w;            // local window
  int stage;        // 0 created, 1 profiled, 2 compacted / decoding
  int steps_done;
  char err[256];
  // optional device-time accounting
  // 0 off; 1 every kernel group; N > 1: the prompt-time phases always, a decode step when
  // its index is a multiple of N
  int timing;
  struct timed { int phase; int a, b; };   // indices into `events`
  std::vector<timed> pending;
  std::vector<hipEvent_t> events;          // recorded since the last read
  std::vector<hipEvent_t> spare;
};

// Tokens per split-KV work item of the decode kernels: 256 for long sequences, 128 when a unit
// can hold at most 4096 tokens (finer items balance short caches better; measured per shape).
inline int fg_decode_chunk(int prompt_len, int max_new_tokens) {
  return ((long long)prompt_len + max_new_tokens <= 4096) ? 128 : 256;
}

// ---------------------------------------------------------------- launch arguments
struct fg_profile_args {
  const void* Q; const void* K;
  float2* rowstat; double* colsum; double* bandcol;
  int U, n, d, w;
  int G;  // query heads per K/V unit: Q and rowstat hold U * G units
  float scale;
};

struct fg_select_args {
  const double* colsum; const double* bandcol; const uint8_t* token_class;  // [B, n]
  uint8_t* keep; int32_t* slot;
  int32_t* policy; double* recov; int32_t* kcount; int32_t* cap; int32_t* len;
  int32_t* policy_out; double* recov_out; int32_t* kcount_out;  // optional caller copies
  int U, n, units_per_seq, w, S, G;
  double T, r_f;
  int forced_policy;
  int family[4];  // FG_COMP_* mask of policy ids 0..3 (0 = unused id)
};

struct fg_compact_args {
  const void* K; const void* V;
  const double* colsum; const uint8_t* keep; const int32_t* slot;   // keep: 0, or 4 | class bits
  const int32_t* cap; int64_t* off; const int32_t* len; int32_t* flags;
  void* ck; void* cv; double* cscore; int32_t* cpos; uint8_t* ccls;
  int U, n, d, esize, units_per_seq;
  int64_t pool_tokens;
};

struct fg_decode_args {
  const void* q; const void* k_new; const void* v_new; const uint8_t* class_new; void* out;
  const int32_t* policy; const int32_t* cap; const int64_t* off; int32_t* len; int32_t* flags;
  void* ck; void* cv; double* cscore; int32_t* cpos; uint8_t* ccls; double* clogit;
  const int32_t* chunk_off; int32_t* item_unit; float* part;
  int U, n, d, dtype, units_per_seq, w, step, G;
  int family[4];   // FG_COMP_* mask of policy ids 0..3 (stability probe)
  double* probe;   // NULL, or [U, 5]: this step's attention mass on every family member
  double r_f;
  float scale;
  int64_t max_chunks;
  int chunk;       // tokens per work item (128 or 256)
};

struct fg_export_args {
  const int64_t* off; const int32_t* len; const int32_t* flags;
  const void* ck; const void* cv; const double* cscore; const int32_t* cpos;
  int32_t* lengths; int64_t* offsets; int32_t* positions; double* scores; void* keys; void* values;
  int32_t* status;
  int U, d, esize, max_pos;  // max_pos = n + S
};

hipError_t fg_launch_profile_bf16(const fg_profile_args&, int pass, hipStream_t);
hipError_t fg_launch_profile_f32(const fg_profile_args&, int pass, hipStream_t);
hipError_t fg_launch_lse_to_rowstat(const float* lse_nat, float2* rowstat, size_t count, hipStream_t);
constexpr int FG_MAX_CLASS_IDS = 64;  // ids per list of fastgen_classify (passed by value)
struct fg_classify_args {
  const int32_t* token_ids; uint8_t* token_class; long long count;
  int num_special, num_punct;
  int32_t special[FG_MAX_CLASS_IDS], punct[FG_MAX_CLASS_IDS];
};
hipError_t fg_launch_classify(const fg_classify_args&, hipStream_t);
hipError_t fg_launch_select(const fg_select_args&, hipStream_t);
hipError_t fg_launch_compact(const fg_compact_args&, hipStream_t);
hipError_t fg_launch_offsets(const int32_t* cap, const int32_t* len, const int32_t* policy, int64_t* off,
                             int32_t* chunk_off, int32_t* item_unit, int32_t* flags, int U, int64_t pool_tokens,
                             int64_t max_chunks, int chunk, hipStream_t);
hipError_t fg_launch_decode_attn(const fg_decode_args&, hipStream_t);
hipError_t fg_launch_decode_update(const fg_decode_args&, hipStream_t);
hipError_t fg_launch_export(const fg_export_args&, hipStream_t);
