// Gated delta-rule decode step for GDN (scalar gate) and KDA (per-key-channel gate), gfx950.
//
// Appendix B of the paper gives the recurrences
//     GDN:  S_t = alpha_t (I - beta_t k_t k_t^T) S_{t-1} + beta_t k_t v_t^T
//     KDA:  S_t = (I - beta_t k_t k_t^T) diag(alpha_t) S_{t-1} + beta_t k_t v_t^T
// Both are  S_t = Sbar + k delta^T  with Sbar the decayed state, u = Sbar^T k and delta = beta (v - u).
// The read-out  o = scale S_t^T q  equals  scale (Sbar^T q + (k.q) delta),  so both reductions over
// the key dimension run over the decayed OLD state: the tile is read from HBM once, updated in
// registers and written once.
//
// Work split.  Value columns are independent of each other (every formula above acts column by
// column), so a wavefront owns 32 columns and all dk rows and never talks to another wavefront:
// no barrier.  Lane (r8 = lane/8, c8 = lane%8) holds columns 4*c8..4*c8+3 of rows
// r8*dk/8 .. (r8+1)*dk/8-1, i.e. dk/8 float4 registers.  One load instruction of the wavefront
// fetches 8 full 128-byte lines.  The key-dimension sums finish with a 3-step butterfly over r8.
// k, q and KDA's gate vector are fetched once per wavefront, coalesced, and handed to the lanes
// through a few KiB of LDS that only this wavefront touches.
#include "common.h"
#include "delta_step_device.h"

namespace {

// STEPS: 0 = the one-token body, else the tokens per call the multi-token body has room for.  The multi-token body at
// 128x128 is asked to fit four wavefronts per SIMD (it does, without spilling: 110-112 registers).
template <int DK, int DV, bool KDA, int STEPS>
__global__ __launch_bounds__(DV * 2, (DK == 128 && STEPS > 0) ? 4 : 1) void delta_step_kernel(DeltaParams p) {
  __shared__ __attribute__((aligned(16))) float park[delta_park_floats<DK, DV, KDA, STEPS>()];
  delta_step_body<DK, DV, KDA, STEPS>(p, interleaved_tile(blockIdx.x, gridDim.x), blockIdx.x, park);
}

// Tokens per call from which the decode steps run on the chunk-parallel kernels, whose time hardly depends on the
// token count up to 16, while the register-resident body, past the 5 or 6 tokens whose arithmetic hides behind the
// tile's memory traffic, adds 3 (GDN) to 5 us (KDA) per token (measured at batch 64, register-resident against chunked,
// us: GDN 6 tokens 51 against 51.5, 7 tokens 52 against 51, 8 tokens 54.4 against 51.2, 10 tokens 59.6 against 53;
// KDA 6 tokens 51.7 against 66, 7 tokens 54.4 against 62, 8 tokens 61.1 against 61.7, 10 tokens 71 against 63.6).
constexpr int kChunkedFromGdn = 7, kChunkedFromKda = 8;
static_assert(kChunkedFromGdn - 1 <= kMaxRegisterSteps128 && kChunkedFromKda - 1 <= kMaxRegisterSteps128,
              "the register-resident kernel must have room for every call that is not chunked");

}  // namespace

// Checks the arguments of one recurrent step and, when they pass, describes its launch in *launch (if not null).
sa_status sa::delta_prepare(bool kda, const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                            const float* state_in, float* state_out, float* out, const int32_t* slot_idx, const int32_t* req_idx,
                            int n_req, int B, int T, int H, int Hk, int dk, int dv, float scale, int n_commit, const int32_t* n_commit_rows,
                            sa::DeltaLaunch* launch) {
  const char* name = kda ? "kda_decode_step" : "gdn_decode_step";
  if (launch) {
    launch->rows = 0;
    launch->chunked = false;
  }
  static_assert(kMaxRegisterSteps64 == 16, "the entry points admit up to 16 tokens per call");
  SA_REQUIRE(B >= 0 && T >= 1 && T <= 16, SA_EINVAL, "%s: need B >= 0 and 1 <= T <= 16 (B=%d, T=%d)", name, B, T);
  SA_REQUIRE(H >= 1 && Hk >= 1 && H % Hk == 0, SA_EINVAL, "%s: H must be a positive multiple of Hk (H=%d, Hk=%d)", name, H, Hk);
  SA_REQUIRE(n_commit >= 0 && n_commit <= T, SA_EINVAL, "%s: n_commit=%d outside [0,T=%d]", name, n_commit, T);
  SA_REQUIRE((dk == 64 && dv == 64) || (dk == 128 && dv == 128), SA_EUNSUPPORTED,
             "%s: (dk,dv)=(%d,%d) not in {(64,64),(128,128)}", name, dk, dv);
  const int rows = req_idx ? n_req : B;
  SA_REQUIRE(rows >= 0 && rows <= B, SA_EINVAL, "%s: n_req=%d outside [0,B=%d]", name, n_req, B);
  if (rows == 0) return SA_OK;
  SA_REQUIRE(q && k && v && alpha && beta && state_in && state_out && out, SA_EINVAL, "%s: null pointer", name);
  SA_REQUIRE(sa::aligned(q, 16) && sa::aligned(k, 16) && sa::aligned(v, 16) && sa::aligned(state_in, 16) &&
                 sa::aligned(state_out, 16) && sa::aligned(out, 16) && sa::aligned(alpha, kda ? 16 : 4) &&
                 sa::aligned(beta, 4) && sa::aligned(slot_idx, 4) && sa::aligned(req_idx, 4) && sa::aligned(n_commit_rows, 4),
             SA_EINVAL, "%s: misaligned pointer", name);
  SA_REQUIRE(static_cast<long long>(rows) * H <= 0x7fffffffLL, SA_EUNSUPPORTED, "%s: too many tiles", name);
  // Longer calls run on the chunk-parallel kernels: they take the same arguments and write the same state for any n_commit.
  if (dk == 128 && T >= (kda ? kChunkedFromKda : kChunkedFromGdn)) {
    if (launch) launch->chunked = true;
    return sa::chunked_steps(kda, true, name, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk,
                             dv, scale, n_commit, n_commit_rows, nullptr);
  }
  if (!launch) return SA_OK;
  launch->p = DeltaParams{static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v),
                          alpha, beta, state_in, state_out, out, slot_idx, req_idx, T, H, Hk, scale, n_commit, n_commit_rows};
  launch->rows = rows;
  return SA_OK;
}

namespace {

template <bool KDA>
sa_status step_launch(bool dry_run, const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                      const float* state_in, float* state_out, float* out, const int32_t* slot_idx, const int32_t* req_idx,
                      int n_req, int B, int T, int H, int Hk, int dk, int dv, float scale, int n_commit, const int32_t* n_commit_rows,
                      void* stream) {
  const char* name = KDA ? "kda_decode_step" : "gdn_decode_step";
  sa::DeltaLaunch l;
  sa_status st = sa::delta_prepare(KDA, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk, dv,
                                   scale, n_commit, n_commit_rows, &l);
  if (st != SA_OK || dry_run) return st;
  if (l.chunked)
    return sa::chunked_steps(KDA, false, name, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk,
                             dv, scale, n_commit, n_commit_rows, stream);
  if (l.rows == 0) return SA_OK;
  const DeltaParams& p = l.p;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid(static_cast<unsigned>(l.rows * H));
  const int kid = KDA ? SA_K_KDA : SA_K_GDN;
  const bool single = T == 1 && n_commit == 1 && !n_commit_rows;
  if (dk == 128 && single)
    sa::launch(kid, delta_step_kernel<128, 128, KDA, 0>, grid, dim3(256), 0, s, p);
  else if (dk == 128)
    sa::launch(kid, delta_step_kernel<128, 128, KDA, kMaxRegisterSteps128>, grid, dim3(256), 0, s, p);
  else if (single)
    sa::launch(kid, delta_step_kernel<64, 64, KDA, 0>, grid, dim3(128), 0, s, p);
  else
    sa::launch(kid, delta_step_kernel<64, 64, KDA, kMaxRegisterSteps64>, grid, dim3(128), 0, s, p);
  return sa::check_launch(name);
}

}  // namespace

extern "C" sa_status gdn_decode_step(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                                     const float* state_in, float* state_out, float* out, const int32_t* slot_idx,
                                     const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv,
                                     float scale, int n_commit, void* stream) {
  return step_launch<false>(false, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B,
                       T, H, Hk, dk, dv, scale, n_commit, nullptr, stream);
}

extern "C" sa_status kda_decode_step(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                                     const float* state_in, float* state_out, float* out, const int32_t* slot_idx,
                                     const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv,
                                     float scale, int n_commit, void* stream) {
  return step_launch<true>(false, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T,
                      H, Hk, dk, dv, scale, n_commit, nullptr, stream);
}

// The same steps with the committed prefix chosen per request (self-speculative decoding: every request accepts
// its own number of drafted tokens).
extern "C" sa_status gdn_decode_step_var(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                                         const float* state_in, float* state_out, float* out, const int32_t* slot_idx,
                                         const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv,
                                         float scale, const int32_t* n_commit_rows, void* stream) {
  SA_REQUIRE(n_commit_rows || B == 0, SA_EINVAL, "gdn_decode_step_var: n_commit_rows is null");
  return step_launch<false>(false, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk, dv,
                            scale, 0, n_commit_rows, stream);
}

extern "C" sa_status kda_decode_step_var(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                                         const float* state_in, float* state_out, float* out, const int32_t* slot_idx,
                                         const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv,
                                         float scale, const int32_t* n_commit_rows, void* stream) {
  SA_REQUIRE(n_commit_rows || B == 0, SA_EINVAL, "kda_decode_step_var: n_commit_rows is null");
  return step_launch<true>(false, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk, dk, dv,
                           scale, 0, n_commit_rows, stream);
}
