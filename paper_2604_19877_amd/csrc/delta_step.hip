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
// no LDS, no barrier.  Lane (r8 = lane/8, c8 = lane%8) holds columns 4*c8..4*c8+3 of rows
// r8*dk/8 .. (r8+1)*dk/8-1, i.e. dk/8 float4 registers.  One load instruction of the wavefront
// fetches 8 full 128-byte lines.  The key-dimension sums finish with a 3-step butterfly over r8.
#include "common.h"
#include "delta_device.h"

namespace {

struct DeltaParams {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  const float* alpha;
  const float* beta;
  const float* state_in;
  float* state_out;
  float* out;
  const int32_t* slot_idx;
  const int32_t* req_idx;
  int T, H, Hk;
  float scale;
  int n_commit;
};

// Operands of one step as they arrive from memory (bf16 still packed).
template <int RPL>
struct StepOperands {
  uint4 k[RPL / 8], q[RPL / 8];
  float alpha, beta;  // alpha: the scalar gate of GDN (KDA's gate vector is fetched apart)
  uint2 v;
};

template <int DK, int DV, bool KDA>
__device__ __forceinline__ void load_operands(StepOperands<DK / 8>& o, const DeltaParams& p, size_t bt, int h, int hk, int row0,
                                              int col0) {
  constexpr int RPL = DK / 8;
  const uint4* kp = reinterpret_cast<const uint4*>(p.k + (bt * p.Hk + hk) * DK + row0);
  const uint4* qp = reinterpret_cast<const uint4*>(p.q + (bt * p.Hk + hk) * DK + row0);
#pragma unroll
  for (int i = 0; i < RPL / 8; ++i) {
    o.k[i] = kp[i];
    o.q[i] = qp[i];
  }
  o.v = *reinterpret_cast<const uint2*>(p.v + (bt * p.H + h) * DV + col0);
  o.beta = load_uniform(p.beta, bt * p.H + h);
  o.alpha = KDA ? 1.f : load_uniform(p.alpha, bt * p.H + h);
}

// KDA's gates of this lane's rows for one step.
template <int DK>
__device__ __forceinline__ void load_gate_vector(float4 (&a)[DK / 32], const DeltaParams& p, size_t bt, int h, int row0) {
  const float4* ap = reinterpret_cast<const float4*>(p.alpha + (bt * p.H + h) * DK + row0);
#pragma unroll
  for (int i = 0; i < DK / 32; ++i) a[i] = ap[i];
}

template <int N>
__device__ __forceinline__ void unpack_bf16(const uint4 (&src)[N / 8], float (&dst)[N]) {
#pragma unroll
  for (int i = 0; i < N / 8; ++i) {
    const uint32_t w[4] = {src[i].x, src[i].y, src[i].z, src[i].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      dst[8 * i + 2 * e] = bf16_lo(w[e]);
      dst[8 * i + 2 * e + 1] = bf16_hi(w[e]);
    }
  }
}

// MULTI = false: exactly one committed step (T == 1, n_commit == 1), the decode hot path, with an
// unconditional store.  MULTI = true: any T and n_commit with the tile held in registers; the
// operands of step t+1 are requested before step t is computed.
template <int DK, int DV, bool KDA, bool MULTI>
__global__ __launch_bounds__(DV * 2, (KDA && MULTI && DV == 128) ? 3 : 1) void delta_step_kernel(DeltaParams p) {
  constexpr int RPL = DK / 8;  // rows per lane
  const int r = blockIdx.x / p.H;
  const int h = blockIdx.x - r * p.H;
  const int b = p.req_idx ? p.req_idx[r] : r;
  const int slot = p.slot_idx ? p.slot_idx[b] : b;
  const int hk = h / (p.H / p.Hk);
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int c8 = lane & 7, r8 = lane >> 3;
  const int row0 = r8 * RPL;
  const int col0 = wave * 32 + c8 * 4;
  const int T = MULTI ? p.T : 1;

  const size_t tile = (static_cast<size_t>(slot) * p.H + h) * (DK * DV);
  const float* sin = p.state_in + tile + static_cast<size_t>(row0) * DV + col0;
  float* sout = p.state_out + tile + static_cast<size_t>(row0) * DV + col0;

  // All requests first: the small operands of step 0, then the 16 state rows of this lane.  The
  // scheduling barrier keeps the compiler from sinking any of them towards its first use, which
  // would put a full memory latency on the critical path of every tile.
  StepOperands<RPL> cur, nxt;
  float4 gate_vec[RPL / 4];  // KDA only: single-buffered, the next step's is requested as soon as this step's is applied
  load_operands<DK, DV, KDA>(cur, p, static_cast<size_t>(b) * T, h, hk, row0, col0);
  if constexpr (KDA) load_gate_vector<DK>(gate_vec, p, static_cast<size_t>(b) * T, h, row0);
  float4 s[RPL];
#pragma unroll
  for (int m = 0; m < RPL; ++m) s[m] = load_state(sin + m * DV);
  __builtin_amdgcn_sched_barrier(0);

  if (MULTI && p.n_commit == 0 && p.state_out != p.state_in) {
#pragma unroll
    for (int m = 0; m < RPL; ++m) store_state(sout + m * DV, s[m]);
  }

  for (int t = 0; t < T; ++t) {
    const size_t bt = static_cast<size_t>(b) * T + t;
    if constexpr (MULTI) {
      if (t + 1 < T) load_operands<DK, DV, KDA>(nxt, p, bt + 1, h, hk, row0, col0);
      __builtin_amdgcn_sched_barrier(0);
    }
    float kf[RPL], qf[RPL];
    unpack_bf16<RPL>(cur.k, kf);
    unpack_bf16<RPL>(cur.q, qf);
    const float beta = cur.beta;

    if constexpr (KDA) {
#pragma unroll
      for (int i = 0; i < RPL / 4; ++i) {
        const float4 a = gate_vec[i];
        const float av[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float4& x = s[4 * i + e];
          x.x *= av[e];
          x.y *= av[e];
          x.z *= av[e];
          x.w *= av[e];
        }
      }
      if constexpr (MULTI) {
        if (t + 1 < T) load_gate_vector<DK>(gate_vec, p, bt + 1, h, row0);
      }
    } else {
      const float a = cur.alpha;
#pragma unroll
      for (int m = 0; m < RPL; ++m) {
        s[m].x *= a;
        s[m].y *= a;
        s[m].z *= a;
        s[m].w *= a;
      }
    }

    float4 u = {0.f, 0.f, 0.f, 0.f}, w = {0.f, 0.f, 0.f, 0.f};
    float kq = 0.f;
#pragma unroll
    for (int m = 0; m < RPL; ++m) {
      u.x = fmaf(s[m].x, kf[m], u.x);
      u.y = fmaf(s[m].y, kf[m], u.y);
      u.z = fmaf(s[m].z, kf[m], u.z);
      u.w = fmaf(s[m].w, kf[m], u.w);
      w.x = fmaf(s[m].x, qf[m], w.x);
      w.y = fmaf(s[m].y, qf[m], w.y);
      w.z = fmaf(s[m].z, qf[m], w.z);
      w.w = fmaf(s[m].w, qf[m], w.w);
      kq = fmaf(kf[m], qf[m], kq);
    }
    u.x = reduce_r8(u.x);
    u.y = reduce_r8(u.y);
    u.z = reduce_r8(u.z);
    u.w = reduce_r8(u.w);
    w.x = reduce_r8(w.x);
    w.y = reduce_r8(w.y);
    w.z = reduce_r8(w.z);
    w.w = reduce_r8(w.w);
    kq = reduce_r8(kq);

    float4 d;
    d.x = beta * (bf16_lo(cur.v.x) - u.x);
    d.y = beta * (bf16_hi(cur.v.x) - u.y);
    d.z = beta * (bf16_lo(cur.v.y) - u.z);
    d.w = beta * (bf16_hi(cur.v.y) - u.w);
#pragma unroll
    for (int m = 0; m < RPL; ++m) {
      s[m].x = fmaf(kf[m], d.x, s[m].x);
      s[m].y = fmaf(kf[m], d.y, s[m].y);
      s[m].z = fmaf(kf[m], d.z, s[m].z);
      s[m].w = fmaf(kf[m], d.w, s[m].w);
    }
    if (!MULTI || t + 1 == p.n_commit) {
#pragma unroll
      for (int m = 0; m < RPL; ++m) store_state(sout + m * DV, s[m]);
    }
    if (r8 == 0) {
      float4 o;
      o.x = p.scale * fmaf(kq, d.x, w.x);
      o.y = p.scale * fmaf(kq, d.y, w.y);
      o.z = p.scale * fmaf(kq, d.z, w.z);
      o.w = p.scale * fmaf(kq, d.w, w.w);
      *reinterpret_cast<float4*>(p.out + (bt * p.H + h) * DV + col0) = o;
    }
    if constexpr (MULTI) cur = nxt;
  }
}

constexpr int kChunkedFrom = 5;  // tokens per call from which the decode steps run on the chunk-parallel kernels

template <bool KDA>
sa_status step_launch(bool dry_run, const char* name, const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                 const float* state_in, float* state_out, float* out, const int32_t* slot_idx, const int32_t* req_idx,
                 int n_req, int B, int T, int H, int Hk, int dk, int dv, float scale, int n_commit, void* stream) {
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
                 sa::aligned(state_out, 16) && sa::aligned(out, 16) && sa::aligned(alpha, KDA ? 16 : 4) &&
                 sa::aligned(beta, 4) && sa::aligned(slot_idx, 4) && sa::aligned(req_idx, 4),
             SA_EINVAL, "%s: misaligned pointer", name);
  SA_REQUIRE(static_cast<long long>(rows) * H <= 0x7fffffffLL, SA_EUNSUPPORTED, "%s: too many tiles", name);
  // From 5 tokens per call the chunk-parallel kernels are faster at 128x128 (8 tokens: 56 / 62 us against
  // 66 / 74 us); they take the same arguments and write the same state for any n_commit.
  if (dk == 128 && T >= kChunkedFrom)
    return sa::chunked_steps(KDA, dry_run, name, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H,
                             Hk, dk, dv, scale, n_commit, stream);
  if (dry_run) return SA_OK;

  DeltaParams p{static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v),
                alpha, beta, state_in, state_out, out, slot_idx, req_idx, T, H, Hk, scale, n_commit};
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid(static_cast<unsigned>(rows * H));
  const int kid = KDA ? SA_K_KDA : SA_K_GDN;
  const bool single = T == 1 && n_commit == 1;
  if (dk == 128 && single)
    sa::launch(kid, delta_step_kernel<128, 128, KDA, false>, grid, dim3(256), 0, s, p);
  else if (dk == 128)
    sa::launch(kid, delta_step_kernel<128, 128, KDA, true>, grid, dim3(256), 0, s, p);
  else if (single)
    sa::launch(kid, delta_step_kernel<64, 64, KDA, false>, grid, dim3(128), 0, s, p);
  else
    sa::launch(kid, delta_step_kernel<64, 64, KDA, true>, grid, dim3(128), 0, s, p);
  return sa::check_launch(name);
}

}  // namespace

extern "C" sa_status gdn_decode_step(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                                     const float* state_in, float* state_out, float* out, const int32_t* slot_idx,
                                     const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv,
                                     float scale, int n_commit, void* stream) {
  return step_launch<false>(false, "gdn_decode_step", q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B,
                       T, H, Hk, dk, dv, scale, n_commit, stream);
}

extern "C" sa_status kda_decode_step(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                                     const float* state_in, float* state_out, float* out, const int32_t* slot_idx,
                                     const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv,
                                     float scale, int n_commit, void* stream) {
  return step_launch<true>(false, "kda_decode_step", q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T,
                      H, Hk, dk, dv, scale, n_commit, stream);
}

// Argument check of a recurrent step without enqueueing anything (used by placement_decode to validate a
// whole stack before its first launch).
sa_status sa::check_recurrent_step(bool kda, const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                                   const float* state_in, float* state_out, float* out, const int32_t* slot_idx,
                                   const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv, int n_commit) {
  if (kda)
    return step_launch<true>(true, "kda_decode_step", q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H,
                        Hk, dk, dv, 1.f, n_commit, nullptr);
  return step_launch<false>(true, "gdn_decode_step", q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H,
                       Hk, dk, dv, 1.f, n_commit, nullptr);
}
