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
constexpr int kMaxRegisterSteps128 = 8, kMaxRegisterSteps64 = 16;

// The per-step scalars and value columns of a lane as they arrive from memory (bf16 still packed).
struct StepOperands {
  float alpha, beta;  // alpha: the scalar gate of GDN (KDA's gate vector goes through LDS)
  uint2 v;
};

template <int DV, bool KDA>
__device__ __forceinline__ void load_operands(StepOperands& o, const DeltaParams& p, size_t bt, int h, int col0) {
  o.v = *reinterpret_cast<const uint2*>(p.v + (bt * p.H + h) * DV + col0);
  o.beta = load_uniform(p.beta, bt * p.H + h);
  o.alpha = KDA ? 1.f : load_uniform(p.alpha, bt * p.H + h);
}

// How a wavefront parks one step's key-dimension vector (k, q or KDA's gates; DK fp32 values) in LDS for its lanes.
// The 8 lane groups r8 each own RPL = DK/8 consecutive rows; group r8's values sit at [r8 * kGroupStride, + RPL) in the
// order the group's lanes keep their rows in registers: position m holds row (m + rot) mod RPL.  A lane then reads its
// RPL values as RPL/4 aligned 16-byte loads, whatever `rot` is.  The stride leaves 4 floats between groups so that
// the 8 groups' 16-byte reads fall into 8 different sets of 4 banks.
template <int DK>
struct KeyVecLds {
  static constexpr int RPL = DK / 8;
  static constexpr int kGroupStride = RPL + 4;
  static constexpr int kFloats = 8 * kGroupStride;
  // where the value of key row `row` goes
  static __device__ __forceinline__ int slot(int row, int rot) {
    return (row / RPL) * kGroupStride + ((row - rot) & (RPL - 1));
  }
};

// Floats of LDS one workgroup of delta_step_body needs for the parked k, q (and gate) vectors.
// STEPS = 0: the one-token body, a copy per wavefront (so that no barrier is needed); otherwise the multi-token body
// with room for STEPS tokens per call, one copy for the workgroup.
template <int DK, int DV, bool KDA, int STEPS>
constexpr int delta_park_floats() {
  return (STEPS ? STEPS : DV / 32) * (KDA ? 3 : 2) * KeyVecLds<DK>::kFloats;
}

// STEPS = 0: exactly one committed step (T == 1, n_commit == 1), the decode hot path, with an
// unconditional store.  STEPS > 0: any T <= STEPS and any n_commit with the tile held in registers; the
// operands of step t+1 are requested before step t is computed.  Its registers do not depend on STEPS (the loop over
// the steps is not unrolled; k, q and the gates wait in LDS), and at 128x128 it runs four wavefronts per SIMD like the
// one-token body.
// The work of one workgroup (2*DV threads): tile `block` = (row of the request list) * H + head.  park_lds: 16-byte
// aligned LDS of delta_park_floats<DK, DV, KDA, STEPS>() floats.
// EITHER (with KDA): one body for both mixers, for kernels whose workgroups run tiles of either kind: a tile with
// scalar_gate set is a GDN tile, whose one gate is written to all key rows of the parked gate vector; everything after
// the fetch is the same code, so such a kernel carries one tile body (and its registers) instead of two.
template <int DK, int DV, bool KDA, int STEPS, bool EITHER = false>
__device__ __forceinline__ void delta_step_body(const DeltaParams& p, const int block, const int start, float* const park_lds,
                                                const bool scalar_gate = false) {
  static_assert(!EITHER || KDA, "the body for either mixer is the per-channel one");
  constexpr bool MULTI = STEPS > 0;
  constexpr int RPL = DK / 8;  // rows per lane
  using Park = KeyVecLds<DK>;
  // Register m of a lane holds row (m + rot) mod RPL of the lane's rows: workgroups launched next to each other start
  // their walk over the tile at different rows, so that at any moment they are not all fetching (and later storing) the
  // same 512-byte slice of their tiles (all tiles are 64 KiB apart, so those slices would all sit on the same few memory
  // channels).  k, q and the gates reach the lanes through LDS already in that rotated order, so any rotation costs the
  // same; four starting rows a quarter of the lane's rows apart measured best (batch 64 / 256, us per step: no rotation
  // 47.0 / 183, these four 44.2 / 173.5, all sixteen rows 45.7 / 176, eight 44.9 / 176, the sixteen in bit-swapped
  // order 44.2 / 176).
  const int rot = (RPL / 4) * (start & 3);
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
  // Where register m's row of this lane sits.  The multi-token body addresses the tile as a base that is the same for
  // the whole workgroup (scalar registers) plus one 32-bit lane offset, and forms the store offsets again where the
  // stores are (the offset passes through an empty asm statement there), so that no address is held across the steps:
  // 64-bit addresses of 16 rows, twice, are what kept it from four wavefronts per SIMD.  The one-token body has the
  // registers and runs 3 % faster with plain per-row pointers (44.1 against 45.6 us at batch 64).
  const float* const tile_in = p.state_in + tile;
  float* const tile_out = p.state_out + tile;
  const uint32_t lane_bytes = static_cast<uint32_t>(row0 * DV + col0) * 4u;
  const auto row_bytes = [rot](int m) { return static_cast<uint32_t>(((m + rot) & (RPL - 1)) * DV) * 4u; };
  const float* const lane_in = tile_in + static_cast<size_t>(row0) * DV + col0;
  float* const lane_out = tile_out + static_cast<size_t>(row0) * DV + col0;
  const auto in_at = [=](uint32_t lane_off, int m) {
    if constexpr (MULTI)
      return reinterpret_cast<const float*>(reinterpret_cast<const char*>(tile_in) + (lane_off + row_bytes(m)));
    else
      return lane_in + ((m + rot) & (RPL - 1)) * DV;
  };
  const auto out_at = [=](uint32_t lane_off, int m) {
    if constexpr (MULTI)
      return reinterpret_cast<float*>(reinterpret_cast<char*>(tile_out) + (lane_off + row_bytes(m)));
    else
      return lane_out + ((m + rot) & (RPL - 1)) * DV;
  };

  // All requests first: the small operands of step 0, then the RPL state rows of this lane.  The
  // scheduling barrier keeps the compiler from sinking any of them towards its first use, which
  // would put a full memory latency on the critical path of every tile.
  StepOperands cur, nxt;
  load_operands<DV, KDA>(cur, p, static_cast<size_t>(b) * T, h, col0);
  // k and q (and KDA's gate vectors) are fetched coalesced (DK values each per step) and parked as fp32 in LDS; a step
  // then reads its lane's rows from there.  Per-lane global loads would fetch each value 32 times over (8 lanes and 4
  // wavefronts share a row): as many load instructions per 4 steps as the state tile itself takes.
  // One-token body: every wavefront fetches and parks its own copy, which no other wavefront reads: no barrier.
  // Multi-token body: one copy for the workgroup, wavefront w fetching steps w, w + (number of wavefronts), ..., and one
  // barrier per call; a copy per wavefront of 8 steps' vectors would leave LDS for two workgroups per CU only.
  constexpr int kWaves = DV / 32;
  constexpr int kVecs = KDA ? 3 : 2;  // k, q, gates
  constexpr int kMine = MULTI ? (STEPS + kWaves - 1) / kWaves : 1;  // steps this wavefront fetches
  static_assert(delta_park_floats<DK, DV, KDA, STEPS>() == (MULTI ? STEPS : kWaves) * kVecs * Park::kFloats);
  float* const my_park = MULTI ? park_lds : park_lds + wave * (kVecs * Park::kFloats);
  const auto fetched_step = [wave](int i) { return MULTI ? wave + i * kWaves : 0; };
  float2 gate_fetch[KDA ? kMine : 1];
  uint32_t k_fetch[kMine], q_fetch[kMine];
  {
    const uint32_t* const ksrc = reinterpret_cast<const uint32_t*>(p.k + (static_cast<size_t>(b) * T * p.Hk + hk) * DK);
    const uint32_t* const qsrc = reinterpret_cast<const uint32_t*>(p.q + (static_cast<size_t>(b) * T * p.Hk + hk) * DK);
    const size_t step_words = static_cast<size_t>(p.Hk) * DK / 2;
#pragma unroll
    for (int i = 0; i < kMine; ++i) {
      const int t = fetched_step(i);
      if (t < T) {
        if constexpr (DK == 128) {
          k_fetch[i] = ksrc[t * step_words + lane];
          q_fetch[i] = qsrc[t * step_words + lane];
        } else {  // 32 words each: the lower half of the wavefront fetches k, the upper half q
          k_fetch[i] = (lane < 32 ? ksrc : qsrc)[t * step_words + (lane & 31)];
        }
      }
    }
  }
  if constexpr (KDA) {
    const float* const src = p.alpha + (static_cast<size_t>(b) * T * p.H + h) * DK;
#pragma unroll
    for (int i = 0; i < kMine; ++i) {
      const int t = fetched_step(i);
      if (t < T) {
        if (EITHER && scalar_gate) {
          const float a = load_uniform(p.alpha, (static_cast<size_t>(b) * T + t) * p.H + h);
          gate_fetch[i] = float2{a, a};
        } else if constexpr (DK == 128) {
          gate_fetch[i] = *reinterpret_cast<const float2*>(src + static_cast<size_t>(t) * p.H * DK + 2 * lane);
        } else {
          gate_fetch[i].x = src[static_cast<size_t>(t) * p.H * DK + lane];
        }
      }
    }
  }
  float4 s[RPL];
#pragma unroll
  for (int m = 0; m < RPL; ++m) s[m] = load_state(in_at(lane_bytes, m));
  __builtin_amdgcn_sched_barrier(0);
  {
    // where this lane's fetched values go: DK = 128: rows 2*lane, 2*lane+1 of k, of q and of the gates; DK = 64: rows
    // 2*(lane%32), +1 of k (lower half of the wavefront) or q (upper half), row `lane` of the gates
    const int pair_row = DK == 128 ? 2 * lane : 2 * (lane & 31);
    const int at0 = Park::slot(pair_row, rot), at1 = Park::slot(pair_row + 1, rot);
    const int vec = DK == 128 ? 0 : (lane >> 5) * Park::kFloats;  // DK = 64: the upper half writes into q's vector
#pragma unroll
    for (int i = 0; i < kMine; ++i) {
      const int t = fetched_step(i);
      if (t < T) {
        float* const base = my_park + t * (kVecs * Park::kFloats);
        base[vec + at0] = bf16_lo(k_fetch[i]);
        base[vec + at1] = bf16_hi(k_fetch[i]);
        if constexpr (DK == 128) {
          base[Park::kFloats + at0] = bf16_lo(q_fetch[i]);
          base[Park::kFloats + at1] = bf16_hi(q_fetch[i]);
        }
        if constexpr (KDA) {
          if constexpr (DK == 128) {
            base[2 * Park::kFloats + at0] = gate_fetch[i].x;
            base[2 * Park::kFloats + at1] = gate_fetch[i].y;
          } else {
            base[2 * Park::kFloats + Park::slot(lane, rot)] = gate_fetch[i].x;
          }
        }
      }
    }
    if constexpr (MULTI)
      __syncthreads();  // every wavefront of the workgroup reaches this: the body has no early exit
    else
      wave_lds_sync();
  }

  if (MULTI && n_commit == 0 && p.state_out != p.state_in) {
#pragma unroll
    for (int m = 0; m < RPL; ++m) store_state(out_at(lane_bytes, m), s[m]);
  }

  for (int t = 0; t < T; ++t) {
    const size_t bt = static_cast<size_t>(b) * T + t;
    if constexpr (MULTI) {
      if (t + 1 < T) load_operands<DV, KDA>(nxt, p, bt + 1, h, col0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // this lane's rows of k, q (and the gates) of step t, in register order
    const float* const mine = my_park + t * (kVecs * Park::kFloats) + r8 * Park::kGroupStride;
    const float beta = cur.beta;

    if constexpr (KDA) {
#pragma unroll
      for (int i = 0; i < RPL / 4; ++i) {
        const float4 a = *reinterpret_cast<const float4*>(mine + 2 * Park::kFloats + 4 * i);
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

    // The one-token body reads this lane's k and q from LDS up front (the reads land while the tile's loads are still in
    // flight) and keeps them: it has the registers.  The multi-token body reads them four rows at a time where they
    // are used, and k once more for the update below: held for a whole step they cost 32 registers next to the tile's
    // 64, and with them the body does not fit four wavefronts per SIMD.
    float4 u = {0.f, 0.f, 0.f, 0.f}, w = {0.f, 0.f, 0.f, 0.f};
    float kq = 0.f;
    float k_kept[MULTI ? 1 : RPL], q_kept[MULTI ? 1 : RPL];
    if constexpr (!MULTI) {
#pragma unroll
      for (int j = 0; j < RPL / 4; ++j) {
        const float4 kk = *reinterpret_cast<const float4*>(mine + 4 * j);
        const float4 qq = *reinterpret_cast<const float4*>(mine + Park::kFloats + 4 * j);
        k_kept[4 * j] = kk.x, k_kept[4 * j + 1] = kk.y, k_kept[4 * j + 2] = kk.z, k_kept[4 * j + 3] = kk.w;
        q_kept[4 * j] = qq.x, q_kept[4 * j + 1] = qq.y, q_kept[4 * j + 2] = qq.z, q_kept[4 * j + 3] = qq.w;
      }
    }
#pragma unroll
    for (int j = 0; j < RPL / 4; ++j) {
      float kf[4], qf[4];
      if constexpr (MULTI) {
        const float4 kk = *reinterpret_cast<const float4*>(mine + 4 * j);
        const float4 qq = *reinterpret_cast<const float4*>(mine + Park::kFloats + 4 * j);
        kf[0] = kk.x, kf[1] = kk.y, kf[2] = kk.z, kf[3] = kk.w;
        qf[0] = qq.x, qf[1] = qq.y, qf[2] = qq.z, qf[3] = qq.w;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) kf[e] = k_kept[4 * j + e], qf[e] = q_kept[4 * j + e];
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float4& x = s[4 * j + e];
        u.x = fmaf(x.x, kf[e], u.x);
        u.y = fmaf(x.y, kf[e], u.y);
        u.z = fmaf(x.z, kf[e], u.z);
        u.w = fmaf(x.w, kf[e], u.w);
        w.x = fmaf(x.x, qf[e], w.x);
        w.y = fmaf(x.y, qf[e], w.y);
        w.z = fmaf(x.z, qf[e], w.z);
        w.w = fmaf(x.w, qf[e], w.w);
        kq = fmaf(kf[e], qf[e], kq);
      }
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
      // k again, through an offset the compiler cannot see through (it would otherwise keep the first read's registers)
      int again = 0;
      if constexpr (MULTI) asm volatile("" : "+v"(again));
#pragma unroll
      for (int j = 0; j < RPL / 4; ++j) {
        float kf[4];
        if constexpr (MULTI) {
          const float4 kk = *reinterpret_cast<const float4*>(mine + again + 4 * j);
          kf[0] = kk.x, kf[1] = kk.y, kf[2] = kk.z, kf[3] = kk.w;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) kf[e] = k_kept[4 * j + e];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float4& x = s[4 * j + e];
          x.x = fmaf(kf[e], ds.x, x.x);
          x.y = fmaf(kf[e], ds.y, x.y);
          x.z = fmaf(kf[e], ds.z, x.z);
          x.w = fmaf(kf[e], ds.w, x.w);
        }
      }
    }
    if (!MULTI || t + 1 == n_commit) {
      uint32_t here = lane_bytes;
      if constexpr (MULTI) asm volatile("" : "+v"(here));
#pragma unroll
      for (int m = 0; m < RPL; ++m) {
        float4 x = s[m];
        if constexpr (LAZY) {
          x.x *= carry;
          x.y *= carry;
          x.z *= carry;
          x.w *= carry;
        }
        store_state(out_at(here, m), x);
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
