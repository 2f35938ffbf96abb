// Whole-block decode step of GDN / KDA: causal conv + SiLU, L2 norm, gate activations, the
// delta-rule state update and the gated RMS norm of the read-out in one launch, gfx950.
//
// Appendix B of the paper lists these operations around the recurrence and Section 6 has the decode
// step update the recurrent state and the convolution histories in place; separately they are four
// tiny launches around a 48 us one.  Here the workgroup that owns a 128x128 state tile first requests the
// tile (16 non-temporal loads per lane, in flight during everything that follows), then its 256
// threads compute the 128 q, 128 k and 128 v channels of this head, one channel per thread:
// Kc-tap depthwise convolution over the stored inputs and the new one, SiLU, and the shifted
// convolution state written back by the same thread that read it.  q and k are L2-normalised with a
// wavefront reduction plus one LDS exchange; the activated channels, the per-channel KDA gate and
// the norms reach the lanes through LDS.  The state update is the one of delta_step.hip.  The
// read-out's mean square is reduced over the 4 wavefronts through LDS and the normalised, gated
// output is written by the lanes that hold it.
#include "common.h"
#include "delta_device.h"

namespace {

struct BlockParams {
  sa_block_io io;
  const float* state_in;
  float* state_out;
  float* out;
  const int32_t* slot_idx;
  const int32_t* req_idx;
  int H, Hk;
  float scale;
};

__device__ __forceinline__ float silu(float x) { return x / (1.f + __expf(-x)); }
__device__ __forceinline__ float sigmoidf(float x) { return 1.f / (1.f + __expf(-x)); }
__device__ __forceinline__ float softplusf(float x) { return x > 20.f ? x : log1pf(__expf(x)); }

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) x += __shfl_xor(x, m);
  return x;
}

// One channel of a depthwise causal convolution: returns SiLU(w . (history, x)) and shifts the history.
__device__ __forceinline__ float conv_channel(const uint16_t* x, const float* w, const uint16_t* hist_in, uint16_t* hist_out,
                                              size_t C, size_t c, int taps, bool write_back) {
  const uint16_t xn = x[c];
  uint16_t h[3] = {0, 0, 0};
  float acc = w[static_cast<size_t>(taps - 1) * C + c] * __uint_as_float(static_cast<uint32_t>(xn) << 16);
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    if (j < taps - 1) {
      h[j] = hist_in[static_cast<size_t>(j) * C + c];
      acc = fmaf(w[static_cast<size_t>(j) * C + c], __uint_as_float(static_cast<uint32_t>(h[j]) << 16), acc);
    }
  }
  if (write_back) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
      if (j + 1 < taps - 1) hist_out[static_cast<size_t>(j) * C + c] = h[j + 1];
    hist_out[static_cast<size_t>(taps - 2) * C + c] = xn;
  }
  return silu(acc);
}

template <int D, bool KDA>
__global__ __launch_bounds__(D * 2) void delta_block_kernel(BlockParams p) {
  constexpr int DK = D, DV = D;
  constexpr int RPL = DK / 8;
  constexpr int WAVES = DV / 32;          // 4 at D = 128; wavefronts [0, WAVES/2) hold q, the rest k
  __shared__ __align__(16) float sh_q[DK], sh_k[DK], sh_v[DV], sh_a[DK];
  __shared__ float sh_sumsq[WAVES], sh_osq[WAVES];

  const sa_block_io& io = p.io;
  const int tile_id = interleaved_tile(blockIdx.x, gridDim.x);
  // register m of a lane holds row (m + turn4) mod RPL of its rows, as in the plain step kernel: neighbouring
  // workgroups do not all fetch the same slice of their tiles at the same moment
  const int turn4 = 4 * (blockIdx.x & (RPL / 4 - 1));
  const int r = tile_id / p.H;
  const int h = tile_id - r * p.H;
  const int b = p.req_idx ? p.req_idx[r] : r;
  const int slot = p.slot_idx ? p.slot_idx[b] : b;
  const int group = p.H / p.Hk;
  const int hk = h / group;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int c8 = lane & 7, r8 = lane >> 3;
  const int row0 = r8 * RPL;
  const int col0 = wave * 32 + c8 * 4;

  const size_t tile = (static_cast<size_t>(slot) * p.H + h) * (DK * DV);
  const float* sin = p.state_in + tile + static_cast<size_t>(row0) * DV + col0;
  float* sout = p.state_out + tile + static_cast<size_t>(row0) * DV + col0;
  float4 s[RPL];
#pragma unroll
  for (int m = 0; m < RPL; ++m) s[m] = load_state(sin + ((m + turn4) & (RPL - 1)) * DV);
  __builtin_amdgcn_sched_barrier(0);

  // ---- pre-processing: one q or k channel and (first half of the threads) one v channel per thread
  const int taps = io.conv_taps;
  const size_t Cqk = static_cast<size_t>(p.Hk) * DK, Cv = static_cast<size_t>(p.H) * DV;
  {
    const bool is_k = tid >= DK;
    const int ch = is_k ? tid - DK : tid;
    const size_t c = static_cast<size_t>(hk) * DK + ch;
    const uint16_t* x = static_cast<const uint16_t*>(is_k ? io.xk : io.xq) + static_cast<size_t>(b) * Cqk;
    const uint16_t* hin = static_cast<const uint16_t*>(is_k ? io.conv_k_in : io.conv_q_in) + static_cast<size_t>(slot) * (taps - 1) * Cqk;
    uint16_t* hout = static_cast<uint16_t*>(is_k ? io.conv_k_out : io.conv_q_out) + static_cast<size_t>(slot) * (taps - 1) * Cqk;
    // with shared key heads every head of the group computes the same channels; the first one stores them
    const float y = conv_channel(x, is_k ? io.wk : io.wq, hin, hout, Cqk, c, taps, h == hk * group);
    (is_k ? sh_k : sh_q)[ch] = y;
    const float ss = wave_sum(y * y);
    if (lane == 0) sh_sumsq[wave] = ss;
    if (!is_k) {
      const size_t cv = static_cast<size_t>(h) * DV + ch;
      sh_v[ch] = conv_channel(static_cast<const uint16_t*>(io.xv) + static_cast<size_t>(b) * Cv, io.wv,
                              static_cast<const uint16_t*>(io.conv_v_in) + static_cast<size_t>(slot) * (taps - 1) * Cv,
                              static_cast<uint16_t*>(io.conv_v_out) + static_cast<size_t>(slot) * (taps - 1) * Cv, Cv, cv, taps, true);
    } else if (KDA) {
      const float raw = io.alpha_raw[(static_cast<size_t>(b) * p.H + h) * DK + ch] + io.dt_bias[static_cast<size_t>(h) * DK + ch];
      sh_a[ch] = __expf(-__expf(io.A_log[h]) * softplusf(raw));
    }
  }
  // GDN's one gate of this head, formed here with the rest of the pre-processing (the activation's long instruction
  // sequence would otherwise sit in the middle of the update, where the tile's registers are all live)
  float gate_scalar = 1.f;
  if constexpr (!KDA)
    gate_scalar = __expf(-__expf(io.A_log[h]) * softplusf(io.alpha_raw[static_cast<size_t>(b) * p.H + h] + io.dt_bias[h]));
  __syncthreads();

  float qsq = 0.f, ksq = 0.f;
#pragma unroll
  for (int w = 0; w < WAVES / 2; ++w) {
    qsq += sh_sumsq[w];
    ksq += sh_sumsq[WAVES / 2 + w];
  }
  const float qinv = rsqrtf(qsq + 1e-6f), kinv = rsqrtf(ksq + 1e-6f);
  float kf[RPL], qf[RPL];
#pragma unroll
  for (int i = 0; i < RPL; ++i) {
    kf[i] = sh_k[row0 + ((i + turn4) & (RPL - 1))] * kinv;
    qf[i] = sh_q[row0 + ((i + turn4) & (RPL - 1))] * qinv;
  }
  const float4 vv = *reinterpret_cast<const float4*>(&sh_v[col0]);
  const float beta = sigmoidf(io.beta_raw[static_cast<size_t>(b) * p.H + h]);

  if constexpr (KDA) {
#pragma unroll
    for (int m = 0; m < RPL; ++m) {
      const float a = sh_a[row0 + ((m + turn4) & (RPL - 1))];
      s[m].x *= a;
      s[m].y *= a;
      s[m].z *= a;
      s[m].w *= a;
    }
  } else {
    const float a = gate_scalar;
#pragma unroll
    for (int m = 0; m < RPL; ++m) {
      s[m].x *= a;
      s[m].y *= a;
      s[m].z *= a;
      s[m].w *= a;
    }
  }

  // ---- the delta-rule step (see delta_step.hip)
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
  d.x = beta * (vv.x - u.x);
  d.y = beta * (vv.y - u.y);
  d.z = beta * (vv.z - u.z);
  d.w = beta * (vv.w - u.w);
#pragma unroll
  for (int m = 0; m < RPL; ++m) {
    s[m].x = fmaf(kf[m], d.x, s[m].x);
    s[m].y = fmaf(kf[m], d.y, s[m].y);
    s[m].z = fmaf(kf[m], d.z, s[m].z);
    s[m].w = fmaf(kf[m], d.w, s[m].w);
    store_state(sout + ((m + turn4) & (RPL - 1)) * DV, s[m]);
  }

  // ---- gated RMS norm of the read-out (every lane holds the 4 columns of its c8; r8 copies agree)
  float4 o;
  o.x = p.scale * fmaf(kq, d.x, w.x);
  o.y = p.scale * fmaf(kq, d.y, w.y);
  o.z = p.scale * fmaf(kq, d.z, w.z);
  o.w = p.scale * fmaf(kq, d.w, w.w);
  float osq = r8 == 0 ? o.x * o.x + o.y * o.y + o.z * o.z + o.w * o.w : 0.f;
  osq = wave_sum(osq);
  if (lane == 0) sh_osq[wave] = osq;
  __syncthreads();
  if (r8 == 0) {
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) tot += sh_osq[i];
    const float inv = rsqrtf(tot * (1.f / DV) + io.norm_eps);
    const size_t at = (static_cast<size_t>(b) * p.H + h) * DV + col0;
    const uint2 zw = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(io.z) + at);
    const float4 nw = *reinterpret_cast<const float4*>(io.norm_weight + col0);
    const float z[4] = {bf16_lo(zw.x), bf16_hi(zw.x), bf16_lo(zw.y), bf16_hi(zw.y)};
    float g[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) g[e] = io.gate_act == 0 ? silu(z[e]) : sigmoidf(z[e]);
    float4 y;
    y.x = nw.x * o.x * inv * g[0];
    y.y = nw.y * o.y * inv * g[1];
    y.z = nw.z * o.z * inv * g[2];
    y.w = nw.w * o.w * inv * g[3];
    *reinterpret_cast<float4*>(p.out + at) = y;
  }
}

template <bool KDA>
sa_status launch_block(const char* name, const sa_block_io* io, const float* state_in, float* state_out, float* out,
                       const int32_t* slot_idx, const int32_t* req_idx, int n_req, int B, int H, int Hk, int dk, int dv,
                       float scale, void* stream) {
  SA_REQUIRE(io, SA_EINVAL, "%s: io is null", name);
  SA_REQUIRE(B >= 0 && H >= 1 && Hk >= 1 && H % Hk == 0, SA_EINVAL, "%s: need B >= 0 and H a positive multiple of Hk", name);
  SA_REQUIRE((dk == 64 && dv == 64) || (dk == 128 && dv == 128), SA_EUNSUPPORTED,
             "%s: (dk,dv)=(%d,%d) not in {(64,64),(128,128)}", name, dk, dv);
  SA_REQUIRE(io->conv_taps >= 2 && io->conv_taps <= 4, SA_EUNSUPPORTED, "%s: conv_taps=%d outside [2,4]", name, io->conv_taps);
  SA_REQUIRE(io->gate_act == 0 || io->gate_act == 1, SA_EINVAL, "%s: gate_act must be 0 (SiLU) or 1 (sigmoid)", name);
  const int rows = req_idx ? n_req : B;
  SA_REQUIRE(rows >= 0 && rows <= B, SA_EINVAL, "%s: n_req=%d outside [0,B=%d]", name, n_req, B);
  if (rows == 0) return SA_OK;
  SA_REQUIRE(io->xq && io->xk && io->xv && io->wq && io->wk && io->wv && io->conv_q_in && io->conv_k_in && io->conv_v_in &&
                 io->conv_q_out && io->conv_k_out && io->conv_v_out && io->beta_raw && io->alpha_raw && io->A_log &&
                 io->dt_bias && io->z && io->norm_weight && state_in && state_out && out,
             SA_EINVAL, "%s: null pointer", name);
  SA_REQUIRE(sa::aligned(state_in, 16) && sa::aligned(state_out, 16) && sa::aligned(out, 16) && sa::aligned(io->z, 8) &&
                 sa::aligned(io->norm_weight, 16) && sa::aligned(io->xq, 2) && sa::aligned(io->xk, 2) && sa::aligned(io->xv, 2) &&
                 sa::aligned(io->wq, 4) && sa::aligned(io->wk, 4) && sa::aligned(io->wv, 4) && sa::aligned(io->beta_raw, 4) &&
                 sa::aligned(io->alpha_raw, 4) && sa::aligned(io->A_log, 4) && sa::aligned(io->dt_bias, 4) &&
                 sa::aligned(slot_idx, 4) && sa::aligned(req_idx, 4),
             SA_EINVAL, "%s: misaligned pointer", name);
  SA_REQUIRE(Hk == H || (io->conv_q_out != io->conv_q_in && io->conv_k_out != io->conv_k_in), SA_EINVAL,
             "%s: with Hk < H the q and k convolution states cannot be updated in place", name);
  SA_REQUIRE(static_cast<long long>(rows) * H <= 0x7fffffffLL, SA_EUNSUPPORTED, "%s: too many tiles", name);

  BlockParams p{*io, state_in, state_out, out, slot_idx, req_idx, H, Hk, scale};
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid(static_cast<unsigned>(rows * H));
  const int kid = KDA ? SA_K_KDA_BLOCK : SA_K_GDN_BLOCK;
  if (dk == 128)
    sa::launch(kid, delta_block_kernel<128, KDA>, grid, dim3(256), 0, s, p);
  else
    sa::launch(kid, delta_block_kernel<64, KDA>, grid, dim3(128), 0, s, p);
  return sa::check_launch(name);
}

}  // namespace

extern "C" sa_status gdn_block_decode(const sa_block_io* io, const float* state_in, float* state_out, float* out,
                                      const int32_t* slot_idx, const int32_t* req_idx, int n_req, int B, int H, int Hk,
                                      int dk, int dv, float scale, void* stream) {
  return launch_block<false>("gdn_block_decode", io, state_in, state_out, out, slot_idx, req_idx, n_req, B, H, Hk, dk, dv,
                             scale, stream);
}

extern "C" sa_status kda_block_decode(const sa_block_io* io, const float* state_in, float* state_out, float* out,
                                      const int32_t* slot_idx, const int32_t* req_idx, int n_req, int B, int H, int Hk,
                                      int dk, int dv, float scale, void* stream) {
  return launch_block<true>("kda_block_decode", io, state_in, state_out, out, slot_idx, req_idx, n_req, B, H, Hk, dk, dv,
                            scale, stream);
}
