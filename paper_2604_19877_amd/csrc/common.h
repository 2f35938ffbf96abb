// Internal helpers shared by the translation units of libsamixers (host side only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "samixers.h"

namespace sa {

// Records a formatted message for sa_last_error() and returns `code`.
sa_status fail(sa_status code, const char* fmt, ...);

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Profiling support (see sa_prof_enable): when enabled, a launch carries a start and a stop event
// that the runtime stamps with the kernel's own begin and end, so the recorded duration is the
// kernel's, without the dispatch gaps that events recorded around a launch would include.
bool prof_enabled();
void prof_record(int kernel_id, hipEvent_t start, hipEvent_t stop);

template <typename K, typename... Args>
inline void launch(int kernel_id, K kernel, dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t stream, Args... args) {
  if (prof_enabled()) {
    hipEvent_t start = nullptr, stop = nullptr;
    if (hipEventCreate(&start) == hipSuccess && hipEventCreate(&stop) == hipSuccess) {
      hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, start, stop, 0, args...);
      prof_record(kernel_id, start, stop);
      return;
    }
    if (start) (void)hipEventDestroy(start);
  }
  hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, args...);
}

// Argument checks of the hot entry points that enqueue nothing (same rules, same messages).
sa_status check_attn_decode(const void* q, const void* kpool, const void* vpool, int n_pages, const int32_t* page_table,
                            int max_pages, const int32_t* seq_lens, const int32_t* req_idx, int n_req, float* out, int B, int T,
                            int Hq, int Hkv, int D, int page_size, int max_seq_len, int window, void* workspace,
                            size_t workspace_bytes);

// The chunk-parallel recurrent kernels (16 tokens at a time on the matrix cores), callable under another entry
// point's name; dry_run checks the arguments and enqueues nothing.
sa_status chunked_steps(bool kda, bool dry_run, const char* name, const void* q, const void* k, const void* v, const float* alpha,
                        const float* beta, const float* state_in, float* state_out, float* out, const int32_t* slot_idx,
                        const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv, float scale, int n_commit,
                        const int32_t* n_commit_rows, void* stream);

// Turns the sticky launch error (if any) into a status.
sa_status check_launch(const char* what);

}  // namespace sa

#define SA_REQUIRE(cond, code, ...)                   \
  do {                                                \
    if (!(cond)) return sa::fail((code), __VA_ARGS__); \
  } while (0)
