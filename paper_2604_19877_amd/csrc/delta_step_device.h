// Device side of the one-token (and register-resident multi-token) gated delta-rule step, shared by the
// stand-alone kernels of delta_step.hip and the fused per-layer kernel of layer_fused.hip.
#pragma once
#include "delta_device.h"
#include "samixers.h"

namespace sa {

// Arguments of one recurrent step launch.
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
  const int32_t* n_commit_rows;  // optional, device int32[B]: the committed prefix of each request (clamped to [0,T]); overrides n_commit
};

// One prepared recurrent step: rows = request rows to launch over (0: nothing to do, or the call runs on the
// chunk-parallel kernels, which `chunked` then says).
struct DeltaLaunch {
  DeltaParams p;
  int rows;
  bool chunked;
};

// Argument checks of gdn_decode_step / kda_decode_step; on success with `launch` not null, fills it (defined in
// delta_step.hip).
sa_status delta_prepare(bool kda, const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                        const float* state_in, float* state_out, float* out, const int32_t* slot_idx, const int32_t* req_idx,
                        int n_req, int B, int T, int H, int Hk, int dk, int dv, float scale, int n_commit, const int32_t* n_commit_rows,
                        DeltaLaunch* launch);

}  // namespace sa

namespace {

using sa::DeltaParams;

// Steps per call for which the multi-token tile body has LDS room at 128x128 (longer calls run on the chunk-parallel
// kernels) and at 64x64 (the entry points' limit).
constexpr int kMaxRegisterSteps128 = 6, kMaxRegisterSteps64 = 16;

// Operands of one step as they arrive from memory (bf16 still packed).
template <int RPL>
struct StepOperands {
  uint2 k[RPL / 4], q[RPL / 4];  // chunk j: the 4 rows this lane holds in registers 4j .. 4j+3
  float alpha, beta;  // alpha: the scalar gate of GDN (KDA's gate vector is fetched apart)
  uint2 v;
};

template <int DK, int DV, bool KDA, bool WITH_KQ = true>
__device__ __forceinline__ void load_operands(StepOperands<DK / 8>& o, const DeltaParams& p, size_t bt, int h, int hk, int row0,
                                              int col0, int turn) {
  constexpr int RPL = DK / 8;
  if constexpr (WITH_KQ) {
    const uint2* kp = reinterpret_cast<const uint2*>(p.k + (bt * p.Hk + hk) * DK + row0);
    const uint2* qp = reinterpret_cast<const uint2*>(p.q + (bt * p.Hk + hk) * DK + row0);
#pragma unroll
    for (int j = 0; j < RPL / 4; ++j) {
      o.k[j] = kp[(j + turn) & (RPL / 4 - 1)];
      o.q[j] = qp[(j + turn) & (RPL / 4 - 1)];
    }
  }
  o.v = *reinterpret_cast<const uint2*>(p.v + (bt * p.H + h) * DV + col0);
  o.beta = load_uniform(p.beta, bt * p.H + h);
  o.alpha = KDA ? 1.f : load_uniform(p.alpha, bt * p.H + h);
}

// KDA's gates of this lane's rows for one step.
template <int DK>
__device__ __forceinline__ void load_gate_vector(float4 (&a)[DK / 32], const DeltaParams& p, size_t bt, int h, int row0, int turn) {
  const float4* ap = reinterpret_cast<const float4*>(p.alpha + (bt * p.H + h) * DK + row0);
#pragma unroll
  for (int j = 0; j < DK / 32; ++j) a[j] = ap[(j + turn) & (DK / 32 - 1)];
}

template <int N>
__device__ __forceinline__ void unpack_bf16(const uint2 (&src)[N / 4], float (&dst)[N]) {
#pragma unroll
  for (int j = 0; j < N / 4; ++j) {
    dst[4 * j] = bf16_lo(src[j].x);
    dst[4 * j + 1] = bf16_hi(src[j].x);
    dst[4 * j + 2] = bf16_lo(src[j].y);
    dst[4 * j + 3] = bf16_hi(src[j].y);
  }
}

// MULTI = false: exactly one committed step (T == 1, n_commit == 1), the decode hot path, with an
// unconditional store.  MULTI = true: any T and n_commit with the tile held in registers; the
// operands of step t+1 are requested before step t is computed.
// The work of one workgroup (2*DV threads): tile `block` = (row of the request list) * H + head.
template <int DK, int DV, bool KDA, bool MULTI>
__device__ __forceinline__ void delta_step_body(const DeltaParams& p, const int block, const int start) {
  constexpr int RPL = DK / 8;  // rows per lane
  // Register m of a lane holds row (m + 4 * turn) mod RPL of the lane's rows: workgroups launched next to each other
  // take different turns, so that at any moment they are not all fetching the same 512-byte slice of their tiles
  // (all tiles are 64 KiB apart, so those slices would all sit on the same few memory channels).
  const int turn = start & (RPL / 4 - 1);
  const int r = block / p.H;
  const int h = block - r * p.H;
  const int b = p.req_idx ? p.req_idx[r] : r;
  const int slot = p.slot_idx ? p.slot_idx[b] : b;
  const int hk = h / (p.H / p.Hk);
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int c8 = lane & 7, r8 = lane >> 3;
  const int row0 = r8 * RPL;
  const int col0 = wave * 32 + c8 * 4;
  constexpr bool LAZY = MULTI && !KDA;  // GDN over several tokens: the scalar decay is carried as a common factor
  float carry = 1.f;
  const int T = MULTI ? p.T : 1;
  // the same for the whole workgroup: kept in a scalar register
  const int n_commit =
      !MULTI ? 1 : __builtin_amdgcn_readfirstlane(p.n_commit_rows ? min(max(p.n_commit_rows[b], 0), T) : p.n_commit);

  const size_t tile = (static_cast<size_t>(slot) * p.H + h) * (DK * DV);
  const float* sin = p.state_in + tile + static_cast<size_t>(row0) * DV + col0;
  float* sout = p.state_out + tile + static_cast<size_t>(row0) * DV + col0;

  // All requests first: the small operands of step 0, then the 16 state rows of this lane.  The
  // scheduling barrier keeps the compiler from sinking any of them towards its first use, which
  // would put a full memory latency on the critical path of every tile.
  StepOperands<RPL> cur, nxt;
  float4 gate_vec[RPL / 4];  // KDA, one token per call: this lane's gates straight from memory
  load_operands<DK, DV, KDA, false>(cur, p, static_cast<size_t>(b) * T, h, hk, row0, col0, turn);
  // Several tokens per call: every wavefront fetches k and q (and KDA's gate vectors) of all its steps once, coalesced
  // (DK values each per step), and parks them in a region of LDS of its own; a step then reads its lane's rows from
  // there.  Per-lane global loads would fetch each value 32 times over (8 lanes and 4 wavefronts share a row): as
  // many load instructions per 4 steps as the state tile itself takes, and a second set of operand registers to hide
  // their latency.  No other wavefront reads the region: no barrier.
  constexpr int kGateSteps = !MULTI ? 1 : DK == 128 ? kMaxRegisterSteps128 : kMaxRegisterSteps64;
  constexpr bool kGatesInLds = KDA;
  __shared__ float gate_lds[kGatesInLds ? (DV / 32) * kGateSteps * DK : 1];
  __shared__ uint32_t kq_lds[(DV / 32) * kGateSteps * DK];  // per (wavefront, step): DK/2 words of k, DK/2 of q
  float* const my_gates = gate_lds + (kGatesInLds ? wave * kGateSteps * DK : 0);
  uint32_t* const my_kq = kq_lds + wave * kGateSteps * DK;
  float2 gate_fetch[kGatesInLds ? kGateSteps : 1];
  uint32_t k_fetch[kGateSteps], q_fetch[kGateSteps];
  {
    const uint32_t* const ksrc = reinterpret_cast<const uint32_t*>(p.k + (static_cast<size_t>(b) * T * p.Hk + hk) * DK);
    const uint32_t* const qsrc = reinterpret_cast<const uint32_t*>(p.q + (static_cast<size_t>(b) * T * p.Hk + hk) * DK);
    const size_t step_words = static_cast<size_t>(p.Hk) * DK / 2;
#pragma unroll
    for (int t = 0; t < kGateSteps; ++t) {
      if (t < T) {
        if constexpr (DK == 128) {
          k_fetch[t] = ksrc[t * step_words + lane];
          q_fetch[t] = qsrc[t * step_words + lane];
        } else {  // 32 words each: the lower half of the wavefront fetches k, the upper half q
          k_fetch[t] = (lane < 32 ? ksrc : qsrc)[t * step_words + (lane & 31)];
        }
      }
    }
  }
  if constexpr (kGatesInLds) {
    const float* const src = p.alpha + (static_cast<size_t>(b) * T * p.H + h) * DK;
#pragma unroll
    for (int t = 0; t < kGateSteps; ++t) {
      if (t < T) {
        if constexpr (DK == 128)
          gate_fetch[t] = *reinterpret_cast<const float2*>(src + static_cast<size_t>(t) * p.H * DK + 2 * lane);
        else
          gate_fetch[t].x = src[static_cast<size_t>(t) * p.H * DK + lane];
      }
    }
  } else if constexpr (KDA) {
    load_gate_vector<DK>(gate_vec, p, static_cast<size_t>(b) * T, h, row0, turn);
  }
  float4 s[RPL];
#pragma unroll
  for (int m = 0; m < RPL; ++m) s[m] = load_state(sin + ((m + 4 * turn) & (RPL - 1)) * DV);
  __builtin_amdgcn_sched_barrier(0);
  {
#pragma unroll
    for (int t = 0; t < kGateSteps; ++t) {
      if (t < T) {
        if constexpr (DK == 128) {
          my_kq[t * DK + lane] = k_fetch[t];
          my_kq[t * DK + DK / 2 + lane] = q_fetch[t];
        } else {
          my_kq[t * DK + lane] = k_fetch[t];  // lanes 32..63 hold q words, which sit right behind the k words
        }
        if constexpr (kGatesInLds) {
          if constexpr (DK == 128)
            *reinterpret_cast<float2*>(my_gates + t * DK + 2 * lane) = gate_fetch[t];
          else
            my_gates[t * DK + lane] = gate_fetch[t].x;
        }
      }
    }
    wave_lds_sync();
  }

  if (MULTI && n_commit == 0 && p.state_out != p.state_in) {
#pragma unroll
    for (int m = 0; m < RPL; ++m) store_state(sout + ((m + 4 * turn) & (RPL - 1)) * DV, s[m]);
  }

  for (int t = 0; t < T; ++t) {
    const size_t bt = static_cast<size_t>(b) * T + t;
    if constexpr (MULTI) {
      if (t + 1 < T) load_operands<DK, DV, KDA, false>(nxt, p, bt + 1, h, hk, row0, col0, turn);
      __builtin_amdgcn_sched_barrier(0);
    }
    {
#pragma unroll
      for (int j = 0; j < RPL / 4; ++j) {
        const int word = (row0 + 4 * ((j + turn) & (RPL / 4 - 1))) / 2;
        cur.k[j] = *reinterpret_cast<const uint2*>(my_kq + t * DK + word);
        cur.q[j] = *reinterpret_cast<const uint2*>(my_kq + t * DK + DK / 2 + word);
      }
    }
    float kf[RPL], qf[RPL];
    unpack_bf16<RPL>(cur.k, kf);
    unpack_bf16<RPL>(cur.q, qf);
    const float beta = cur.beta;

    if constexpr (KDA) {
#pragma unroll
      for (int i = 0; i < RPL / 4; ++i) {
        const float4 a = kGatesInLds ? *reinterpret_cast<const float4*>(my_gates + t * DK + row0 + 4 * ((i + turn) & (RPL / 4 - 1)))
                                     : gate_vec[i];
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
    } else if constexpr (MULTI) {
      // The registers hold the state divided by `carry`, the product of the gates since the last time it was
      // multiplied in: a step then scales the 8 reduced sums and its correction instead of 64 state values.  The
      // gate is the same for the whole workgroup, and so is the decision to multiply the product in (before it
      // could underflow: below 2^-60).
      carry *= cur.alpha;
      if (carry < 8.673617e-19f) {
#pragma unroll
        for (int m = 0; m < RPL; ++m) {
          s[m].x *= carry;
          s[m].y *= carry;
          s[m].z *= carry;
          s[m].w *= carry;
        }
        carry = 1.f;
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

    if constexpr (LAZY) {
      u.x *= carry;
      u.y *= carry;
      u.z *= carry;
      u.w *= carry;
      w.x *= carry;
      w.y *= carry;
      w.z *= carry;
      w.w *= carry;
    }
    float4 d;
    d.x = beta * (bf16_lo(cur.v.x) - u.x);
    d.y = beta * (bf16_hi(cur.v.x) - u.y);
    d.z = beta * (bf16_lo(cur.v.y) - u.z);
    d.w = beta * (bf16_hi(cur.v.y) - u.w);
    {
      // what is added to the registers: the correction over the factor they carry (its reciprocal to 1 ulp)
      float4 ds = d;
      if constexpr (LAZY) {
        const float r = __builtin_amdgcn_rcpf(carry);
        ds.x *= r;
        ds.y *= r;
        ds.z *= r;
        ds.w *= r;
      }
#pragma unroll
      for (int m = 0; m < RPL; ++m) {
        s[m].x = fmaf(kf[m], ds.x, s[m].x);
        s[m].y = fmaf(kf[m], ds.y, s[m].y);
        s[m].z = fmaf(kf[m], ds.z, s[m].z);
        s[m].w = fmaf(kf[m], ds.w, s[m].w);
      }
    }
    if (!MULTI || t + 1 == n_commit) {
#pragma unroll
      for (int m = 0; m < RPL; ++m) {
        float4 x = s[m];
        if constexpr (LAZY) {
          x.x *= carry;
          x.y *= carry;
          x.z *= carry;
          x.w *= carry;
        }
        store_state(sout + ((m + 4 * turn) & (RPL - 1)) * DV, x);
      }
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

}  // namespace
