// Chunk-parallel form of the GDN recurrence on the matrix cores, gfx950: many tokens per state pass.
//
// Appendix B of the paper has GDN evaluated chunk by chunk on a WY representation for long inputs and
// Section 6 uses such kernels for prefill; the paper prints only the token-by-token recurrence
//     S_t = alpha_t (I - beta_t k_t k_t^T) S_{t-1} + beta_t k_t v_t^T,      o_t = scale S_t^T q_t.
// Unrolled over a chunk of C = 16 tokens with g(t,i) = prod_{i<m<=t} alpha_m  (g(t,t) = 1,
// g(t,-1) = the decay from the chunk's start through step t):
//     S_t      = g(t,-1) S_0 + sum_{i<=t} g(t,i) k_i delta_i^T
//     delta_t  = beta_t (v_t - g(t,-1) S_0^T k_t) - sum_{i<t} beta_t g(t,i) (k_t.k_i) delta_i
//     o_t      = scale ( g(t,-1) S_0^T q_t + sum_{i<=t} g(t,i) (q_t.k_i) delta_i )
// so a chunk costs three state-sized matrix products (K S_0, Q S_0, K^T Delta), two 16x16 Gram
// matrices, and one unit-lower-triangular solve with 16 unknown rows.
//
// Precision.  States are fp32 and must stay within 1e-4 of the fp64 recurrence after hundreds of
// steps, so nothing fp32 is rounded to one bf16: every fp32 operand of a matrix product is split into
// several bf16 terms and the product is the sum of one bf16 MFMA per term with fp32 accumulation:
// two terms, each rounded to nearest (relative error 2^-18, unbiased), for the state as an operand
// of K S_0 and Q S_0 and for the corrections delta added to it.  q, k arrive as bf16
// and are used as they are.  The decay factors are applied in fp32 outside the products, as
// 2^(difference of running sums of log2 alpha), which never exceeds 1 (no division, no overflow
// for any alpha in (0,1]).
//
// Work split.  As in the one-token kernel, value columns are independent: a workgroup owns one
// (sequence, head) tile, each of its 4 wavefronts 32 value columns and all 128 key rows.  The
// state lives in registers in the MFMA accumulator layout for the whole call: lane (n = lane%16,
// g = lane/16) holds key rows 16r+4g .. 16r+4g+3 (r = 0..7) of columns 32w+2n and 32w+2n+1.
// That layout is at once the C/D layout of K^T Delta (so the update accumulates in place), the
// B-operand layout of the 16x16x16 product, and - two row tiles side by side, with the A operand
// permuted to match - the B operand of the 16x16x32 product used for K S_0 and Q S_0.
// The workgroup stages each chunk's K and Q in LDS once (token-major for the A operands of
// K S_0 / Q S_0 and the Gram matrices, channel-major for the A operand of K^T Delta), double
// buffered with one barrier per chunk.  Each wavefront solves the triangular system for its own
// columns by 4-row groups: rows live 4 to a lane, so the 4x4 diagonal blocks are eliminated inside
// the lanes (once, for all groups together), and three stages of "broadcast a group's 4 results,
// 4x4 block update in the later groups" finish it.
#include "common.h"
#include "delta_device.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

struct ChunkParams {
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
  int n_commit;  // state_out receives the state after this many tokens (0 .. T)
  const int32_t* n_commit_rows;  // optional, device int32[B]: that count per request (clamped to [0,T]); overrides n_commit
};

constexpr int kD = 128;          // dk = dv
constexpr int kC = 16;           // tokens per chunk
constexpr int kTokRowB = 272;    // bytes of one token row of K or Q in LDS (256 + 16: spreads the rows over banks)
// Channel-major copies of K (16 tokens = 32 bytes per key channel): rows 48 bytes apart plus 8 bytes after every 8
// channels.  They are written 2 bytes at a time by lanes that hold channels 8 apart (each thread stages 8 channels of one
// token) and read 8 bytes at a time by lanes on consecutive channels; with plain 40-byte rows the 16 writing lanes of a
// token fell on 4 LDS banks, with this spacing writers and readers both spread over all banks.
constexpr int kChRowB = 48, kChGroupPadB = 8;
constexpr int kChnB = kD * kChRowB + (kD / 8) * kChGroupPadB;   // bytes of one channel-major copy
__device__ __forceinline__ int chn_row(int channel) { return channel * kChRowB + (channel >> 3) * kChGroupPadB; }
constexpr int kStageB = 2 * kC * kTokRowB + kChnB;  // one chunk's K, Q and transposed K
constexpr int kMatRow = 20;      // floats per row of the per-wavefront 16x16 matrices (16 + 4)
constexpr int kWaveB = (2 * kC * kMatRow + kC * 4) * 4;  // L', M, diagonal blocks of A

// Two-term split with round-to-nearest in both terms: x = hi + lo up to 2^-18 |x|.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pack_rne(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}
struct Split4x2 {
  u32x2 hi, lo;
};
__device__ __forceinline__ Split4x2 split2(const f32x4& x) {
  Split4x2 s;
  s.hi = u32x2{pack_rne(x[0], x[1]), pack_rne(x[2], x[3])};
  const float r0 = x[0] - bf16_lo(s.hi[0]), r1 = x[1] - bf16_hi(s.hi[0]);
  const float r2 = x[2] - bf16_lo(s.hi[1]), r3 = x[3] - bf16_hi(s.hi[1]);
  s.lo = u32x2{pack_rne(r0, r1), pack_rne(r2, r3)};
  return s;
}
__device__ __forceinline__ bf16x8 join8(const u32x2& a, const u32x2& b) {
  return __builtin_bit_cast(bf16x8, u32x4{a[0], a[1], b[0], b[1]});
}

// K^T Delta with Delta as two bf16 terms in ONE 16x16x32 product: the contraction index of the wide instruction
// runs over (token, term), slots 0-3 of a lane's 8 holding tokens 4g..4g+3 with the first term of Delta and
// slots 4-7 the same tokens with the second, so the A operand is the lane's 4 K values twice.
__device__ __forceinline__ f32x4 mfma_two_terms(const u32x2& a, const Split4x2& b, const f32x4& acc) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(join8(a, a), join8(b.hi, b.lo), acc, 0, 0, 0);
}
constexpr int kChRowTile = 16 * kChRowB + 2 * kChGroupPadB;  // bytes from channel c's row to channel c+16's

// 2^x by the bare instruction: results below the smallest normal number come out as 0, which is what the decay
// factors here may do (the library call spends five more instructions on keeping them).
__device__ __forceinline__ float pow2(float x) { return __builtin_amdgcn_exp2f(x); }

// x of the lane D places down the same row of 16 lanes, 0 for the first D lanes of a row.
template <int D>
__device__ __forceinline__ float row_shr(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x110 + D, 0xf, 0xf, true));
}

// The triangular system (I + A) delta = rhs, A = D + L with D the four 4x4 diagonal blocks (a lane holds 4 rows, so a
// block stays inside the lanes of one row group) and L the blocks below them.  Both sides are multiplied by (I + D)^-1
// first: every row group does that 4-row substitution once, at the same time, on its right-hand sides, and the lanes
// that formed L apply it to the column of L they hold.  What remains, (I + L') delta = rhs' with L' = (I + D)^-1 L, is
// solved block row by block row with nothing but broadcasts and 4x4 block updates.
struct DiagBlock {
  f32x4 r1, r2, r3;  // rows 1..3 of this lane's row group's block of D (strictly lower: columns 0..2 are used)
};
__device__ __forceinline__ void diag_solve(f32x4& x, const DiagBlock& d) {
  x[1] = fmaf(-d.r1[0], x[0], x[1]);
  x[2] = fmaf(-d.r2[1], x[1], fmaf(-d.r2[0], x[0], x[2]));
  x[3] = fmaf(-d.r3[2], x[2], fmaf(-d.r3[1], x[1], fmaf(-d.r3[0], x[0], x[3])));
}

// Lane (n, g) brings a[j] = A[4g+j][n] (0 for n >= 4g+j) and m[j] = M[4g+j][n] (0 for n > 4g+j).  Leaves M in m_low
// ([16][kMatRow]), L' in a_off ([16][kMatRow], zero on and above the diagonal blocks) and returns the lane's block of D,
// which went through a_dia ([16][4]).
__device__ __forceinline__ DiagBlock publish_system(const f32x4& a, const f32x4& m, float* a_off, float* m_low, float* a_dia, int n, int g) {
  if ((n >> 2) == g) {
#pragma unroll
    for (int j = 0; j < 4; ++j) a_dia[(4 * g + j) * 4 + (n & 3)] = a[j];
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) m_low[(4 * g + j) * kMatRow + n] = m[j];
  wave_lds_sync();
  DiagBlock d;
  d.r1 = *reinterpret_cast<const f32x4*>(a_dia + (4 * g + 1) * 4);
  d.r2 = *reinterpret_cast<const f32x4*>(a_dia + (4 * g + 2) * 4);
  d.r3 = *reinterpret_cast<const f32x4*>(a_dia + (4 * g + 3) * 4);
  const bool below = (n >> 2) < g;
  f32x4 l = {below ? a[0] : 0.f, below ? a[1] : 0.f, below ? a[2] : 0.f, below ? a[3] : 0.f};
  diag_solve(l, d);
#pragma unroll
  for (int j = 0; j < 4; ++j) a_off[(4 * g + j) * kMatRow + n] = l[j];
  wave_lds_sync();
  return d;
}

// rhs turns into delta in place, for this wavefront's 2 x 16 columns.  Stage gp: the rows of group gp are final; they
// are broadcast and the later groups subtract their block's share (the other groups run the same code on zeros).
__device__ __forceinline__ void solve_rows(f32x4 (&rhs)[2], const float* a_off, const DiagBlock& dia, int n, int g) {
  diag_solve(rhs[0], dia);
  diag_solve(rhs[1], dia);
#pragma unroll
  for (int gp = 0; gp < 3; ++gp) {
    float d[2][4];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int jp = 0; jp < 4; ++jp) d[c][jp] = __shfl(rhs[c][jp], 16 * gp + n);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(a_off + (4 * g + j) * kMatRow + 4 * gp);
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int jp = 0; jp < 4; ++jp) rhs[c][j] = fmaf(-a[jp], d[c][jp], rhs[c][j]);
    }
  }
}

// Read-out: o += M delta on the matrix cores (m_low: [16][kMatRow], zero above the diagonal).  This product
// only reaches the output (tolerance 2e-3), so two rounded terms per operand and the three leading cross
// products are plenty.
__device__ __forceinline__ void readout_rows(f32x4 (&o)[2], const f32x4 (&delta)[2], const float* m_low, int n, int g) {
  const Split4x2 ms = split2(*reinterpret_cast<const f32x4*>(m_low + n * kMatRow + 4 * g));  // A operand: row n, columns 4g..
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    const Split4x2 dl = split2(delta[c]);
    o[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, ms.lo), __builtin_bit_cast(s16x4, dl.hi), o[c], 0, 0, 0);
    o[c] = mfma_two_terms(ms.hi, dl, o[c]);
  }
}

// Writes this lane's part of the state tile (accumulator layout), times `factor`, with the non-temporal hint.  The
// offset is made opaque so that the 32 store addresses are formed here and not kept in registers from the kernel's start.
__device__ __forceinline__ void store_tile(const f32x4 (&S)[8][2], float* sout, uint32_t lane_off, float factor = 1.f) {
  asm volatile("" : "+v"(lane_off));
#pragma unroll
  for (int rt = 0; rt < 8; ++rt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const f32x2 x = {factor * S[rt][0][j], factor * S[rt][1][j]};
      __builtin_nontemporal_store(x, reinterpret_cast<f32x2*>(sout + (lane_off + (16 * rt + j) * kD)));
    }
}

// A value that is the same in every lane, moved to a scalar register.  The empty asm hides where it came from:
// the compiler drops a bare readfirstlane of a value it can prove uniform and then leaves that value in vector registers.
__device__ __forceinline__ int to_scalar(int x) {
  asm volatile("" : "+v"(x));
  return __builtin_amdgcn_readfirstlane(x);
}

// Offsets are formed in bytes in 32 bits so that a load is "scalar base + vector offset".
template <typename V>
__device__ __forceinline__ V load_at(const void* base, uint32_t byte_off) {
  return *reinterpret_cast<const V*>(static_cast<const unsigned char*>(base) + byte_off);
}
// What a thread fetches from global memory for one chunk.
struct ChunkFetch {
  u32x4 kst, qst;     // staging: 8 channels of one token of K and of Q
  uint32_t v[4];      // this lane's two value columns of tokens 4g .. 4g+3
  float alpha, beta;  // of token lane%16
};

// Byte offsets of a thread's loads from the chunk's first token, with tokens past `lim` (the last valid token of
// the chunk) redirected to token `lim`, which is always in bounds.
struct ChunkOffsets {
  uint32_t kq, v[4], gate;
};
__device__ __forceinline__ ChunkOffsets chunk_offsets(const ChunkParams& p, int lim, int col, int g, int n) {
  const int tid = threadIdx.x;
  const int tok = tid >> 4, c8 = (tid & 15) * 8;
  ChunkOffsets o;
  o.kq = (static_cast<uint32_t>(min(tok, lim)) * static_cast<uint32_t>(p.Hk * kD) + c8) * 2u;
  const uint32_t stride = static_cast<uint32_t>(p.H * kD);
#pragma unroll
  for (int j = 0; j < 4; ++j) o.v[j] = (static_cast<uint32_t>(min(4 * g + j, lim)) * stride + col) * 2u;
  o.gate = static_cast<uint32_t>(min(n, lim)) * static_cast<uint32_t>(p.H) * 4u;
  return o;
}

// All addresses are a per-chunk scalar base plus a 32-bit lane offset (a chunk spans < 4 GiB).  The bases advance
// from chunk to chunk by fixed strides.  `offs` holds the offsets of a chunk that lies wholly inside the call, computed
// once per kernel; only the call's last chunk can be ragged, and it overwrites them: tokens past the end are read from
// the last valid token and then replaced by values that leave the state alone: k = q = v = 0, alpha = 1, beta = 0.
// The offsets pass through an empty asm in the block that loads: a load takes the form "scalar base + 32-bit lane
// offset" only when the widening of the offset sits next to it; otherwise the compiler widens the chunk-invariant
// offsets once, keeps them as 64-bit pairs for the whole kernel and adds the chunk's base to each with the vector unit.
struct ChunkBases {
  const uint16_t *k, *q, *v;
  const float *alpha, *beta;
};
__device__ __forceinline__ ChunkBases chunk_bases(const ChunkParams& p, size_t row0, int h, int hk) {
  const size_t kq = (row0 * p.Hk + hk) * kD, base = row0 * p.H + h;
  return ChunkBases{p.k + kq, p.q + kq, p.v + base * kD, p.alpha + base, p.beta + base};
}
__device__ __forceinline__ void next_chunk(ChunkBases& at, const ChunkParams& p) {
  at.k += kC * p.Hk * kD;
  at.q += kC * p.Hk * kD;
  at.v += kC * p.H * kD;
  at.alpha += kC * p.H;
  at.beta += kC * p.H;
}
__device__ __forceinline__ void opaque(ChunkOffsets& o) {
  asm volatile("" : "+v"(o.kq), "+v"(o.v[0]), "+v"(o.v[1]), "+v"(o.v[2]), "+v"(o.v[3]), "+v"(o.gate));
}
// A chunk is fetched in two parts, each straight into the registers the previous chunk's values have just left: K and
// Q for staging as soon as the previous chunk is staged (this part also switches `offs` over for a ragged chunk), the
// per-lane values once the previous chunk's right-hand sides are formed.  `lim` is the chunk's last valid token.
__device__ __forceinline__ void fetch_staging(ChunkFetch& f, const ChunkParams& p, const ChunkBases& at, ChunkOffsets& offs, int lim,
                                              int col, int g, int n) {
  const bool ragged = lim < kC - 1;
  if (ragged) {
    // The empty asm, which the offsets below depend on, keeps this a branch: as selects, their multiplications would run in every chunk.
    asm volatile("" : "+s"(lim));
    offs = chunk_offsets(p, lim, col, g, n);
  }
  asm volatile("" : "+v"(offs.kq));
  f.kst = load_at<u32x4>(at.k, offs.kq);
  f.qst = load_at<u32x4>(at.q, offs.kq);
  if (!ragged) return;
  asm volatile("");
  const bool live = (static_cast<int>(threadIdx.x) >> 4) <= lim;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f.kst[e] = live ? f.kst[e] : 0u;
    f.qst[e] = live ? f.qst[e] : 0u;
  }
}
__device__ __forceinline__ void fetch_lane(ChunkFetch& f, const ChunkBases& at, ChunkOffsets& offs, int lim, int g, int n) {
  asm volatile("" : "+v"(offs.v[0]), "+v"(offs.v[1]), "+v"(offs.v[2]), "+v"(offs.v[3]), "+v"(offs.gate));
#pragma unroll
  for (int j = 0; j < 4; ++j) f.v[j] = load_at<uint32_t>(at.v, offs.v[j]);
  f.alpha = load_at<float>(at.alpha, offs.gate);
  f.beta = load_at<float>(at.beta, offs.gate);
  if (lim >= kC - 1) return;
  asm volatile("");  // a branch, not selects
#pragma unroll
  for (int j = 0; j < 4; ++j) f.v[j] = 4 * g + j <= lim ? f.v[j] : 0u;
  f.alpha = n <= lim ? f.alpha : 1.f;
  f.beta = n <= lim ? f.beta : 0.f;
}

// ONE: the call is a single chunk (T <= 16, a verify pass): nothing is prefetched for a next chunk and one staging
// buffer is enough (144 registers, 26 KiB of LDS).  Both forms are held to three wavefronts per SIMD (168 registers),
// which the kernel of many chunks just fits without spilling (41 KiB of LDS; 8 tokens at batch 64: 51 us against 54 us
// with two wavefronts, 512 tokens 10 % faster).
template <bool ONE>
__global__ __launch_bounds__(256, 3) void gdn_chunk_kernel(ChunkParams p) {
  extern __shared__ __align__(16) unsigned char lds[];
  // Every index here is the same for the whole workgroup; saying so keeps every base address in scalar registers
  // (the divisions run on the vector unit and their results stay in vector registers, and everything computed
  // from them with them, unless they are moved across by hand).
  const int r = to_scalar(blockIdx.x / p.H);
  const int h = blockIdx.x - r * p.H;
  const int b = __builtin_amdgcn_readfirstlane(p.req_idx ? p.req_idx[r] : r);
  const int slot = __builtin_amdgcn_readfirstlane(p.slot_idx ? p.slot_idx[b] : b);
  const int n_commit = __builtin_amdgcn_readfirstlane(p.n_commit_rows ? min(max(p.n_commit_rows[b], 0), p.T) : p.n_commit);
  const int hk = to_scalar(h / (p.H / p.Hk));
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int n = lane & 15, g = lane >> 4;
  const int col = wave * 32 + 2 * n;
  const size_t row0 = static_cast<size_t>(b) * p.T;

  float* const wave_mat = reinterpret_cast<float*>(lds + (ONE ? 1 : 2) * kStageB + wave * kWaveB);
  float* const a_off = wave_mat;                      // [16][kMatRow]: A = beta_t g(t,i) k_t.k_i below its diagonal blocks, block-diagonal part eliminated
  float* const m_low = wave_mat + kC * kMatRow;       // [16][kMatRow]: g(t,i) q_t.k_i for i <= t
  float* const a_dia = wave_mat + 2 * kC * kMatRow;   // [16][4]: A for i in t's own group, i < t

  // Uniform tile base plus a 32-bit lane offset, so that addresses cost one register each.
  const size_t tile = (static_cast<size_t>(slot) * p.H + h) * (kD * kD);
  const float* const sin = p.state_in + tile;
  float* const sout = p.state_out + tile;
  const uint32_t lane_off = static_cast<uint32_t>(4 * g * kD + col);

  // Kept in registers for the whole call (the empty asm stops the compiler from recomputing them per chunk).
  ChunkOffsets offs = chunk_offsets(p, kC - 1, col, g, n);
  opaque(offs);
  ChunkBases at = chunk_bases(p, row0, h, hk);
  float* out_at = p.out + (row0 * p.H + h) * kD;   // the current chunk's first output row, this head
  uint32_t out_off = (static_cast<uint32_t>(4 * g * p.H * kD + col)) * 4u;  // bytes from there to token 4g, this lane's columns
  asm volatile("" : "+v"(out_off));
  ChunkFetch cur;
  fetch_staging(cur, p, at, offs, p.T - 1, col, g, n);
  fetch_lane(cur, at, offs, p.T - 1, g, n);
  // S[rt][c][j]: key row 16 rt + 4 g + j, value column col + c.
  f32x4 S[8][2];
#pragma unroll
  for (int rt = 0; rt < 8; ++rt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const f32x2 x = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(sin + (lane_off + (16 * rt + j) * kD)));
      S[rt][0][j] = x[0];
      S[rt][1][j] = x[1];
    }
  __builtin_amdgcn_sched_barrier(0);

  // The registers hold the state divided by 2^c_log: a chunk's decay g(15,-1) goes into that common factor
  // instead of into 64 multiplications per lane, and the factor is multiplied in once it falls below 2^-96
  // (and wherever the state is stored).  The factor is the same for the whole workgroup.
  float c_log = 0.f;
  const int n_chunks = ONE ? 1 : (p.T + kC - 1) / kC;
  for (int ch = 0; ch < n_chunks; ++ch) {
    const int t0 = ch * kC;
    const int n_keep = n_commit - t0;  // tokens of this chunk that the stored state includes, if it is stored here
    if (n_keep == 0 && n_commit < p.T && (t0 > 0 || sout != sin)) store_tile(S, sout, lane_off, exp2f(c_log));
    unsigned char* const stage = lds + (ONE ? 0 : (ch & 1) * kStageB);
    unsigned char* const k_tok = stage;                       // [16 tokens][kTokRowB]
    unsigned char* const q_tok = stage + kC * kTokRowB;
    unsigned char* const k_chn = stage + 2 * kC * kTokRowB;   // 128 channels, channel c at chn_row(c)
    {
      const int tok = tid >> 4, c8 = (tid & 15) * 8;
      *reinterpret_cast<u32x4*>(k_tok + tok * kTokRowB + c8 * 2) = cur.kst;
      *reinterpret_cast<u32x4*>(q_tok + tok * kTokRowB + c8 * 2) = cur.qst;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t w = cur.kst[e >> 1];
        *reinterpret_cast<uint16_t*>(k_chn + chn_row(c8 + e) + tok * 2) = static_cast<uint16_t>((e & 1) ? (w >> 16) : (w & 0xffffu));
      }
    }
    __syncthreads();
    // The buffer written above was last read two chunks ago, and every wavefront has passed the
    // previous chunk's barrier since, so one barrier per chunk is enough.
    const bool more = !ONE && ch + 1 < n_chunks;
    const int lim = p.T - 1 - t0, lim_next = lim - kC;  // last valid token of this chunk and of the next
    const bool whole = lim >= kC - 1;
    if (more) {
      next_chunk(at, p);
      fetch_staging(cur, p, at, offs, lim_next, col, g, n);
    }

    // K S_0 and Q S_0 for this wavefront's 32 columns (rows = tokens 4g+j), and the Gram matrices
    // (lane (n, g) gets k_t.k_n and q_t.k_n for t = 4g+j).  A operands of the 16x16x32 products: token n,
    // key rows {32s+4g..+3, 32s+16+4g..+3}, the same rows as a pair of state tiles holds in this lane.
    f32x4 kk = {0.f, 0.f, 0.f, 0.f}, qk = {0.f, 0.f, 0.f, 0.f};
    f32x4 u[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}, w[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int off = n * kTokRowB + (32 * s + 4 * g) * 2;
      const bf16x8 kf = join8(*reinterpret_cast<const u32x2*>(k_tok + off), *reinterpret_cast<const u32x2*>(k_tok + off + 32));
      const bf16x8 qf = join8(*reinterpret_cast<const u32x2*>(q_tok + off), *reinterpret_cast<const u32x2*>(q_tok + off + 32));
      kk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, kf, kk, 0, 0, 0);
      qk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf, kf, qk, 0, 0, 0);
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const Split4x2 lo_tile = split2(S[2 * s][c]), hi_tile = split2(S[2 * s + 1][c]);
        const bf16x8 b_hi = join8(lo_tile.hi, hi_tile.hi), b_lo = join8(lo_tile.lo, hi_tile.lo);
        u[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, b_lo, u[c], 0, 0, 0);
        w[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf, b_lo, w[c], 0, 0, 0);
        u[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, b_hi, u[c], 0, 0, 0);
        w[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf, b_hi, w[c], 0, 0, 0);
      }
    }

    // Decay factors from the running sum of log2(alpha): every g(t,i) = 2^(L_t - L_i) is at most 1, so no
    // product of gates can overflow or divide by an underflowed one.  Every lane holds alpha and beta of
    // token lane%16; a gate below the smallest normal number acts as that number.
    // Inclusive prefix sum L_n over the 16 lanes of a row with row shifts (a lane without a source adds 0).
    float log_sum = __builtin_amdgcn_logf(fmaxf(cur.alpha, 1.17549435e-38f));  // the bare instruction: its operand is a normal number
    log_sum += row_shr<1>(log_sum);
    log_sum += row_shr<2>(log_sum);
    log_sum += row_shr<4>(log_sum);
    log_sum += row_shr<8>(log_sum);
    const float log_chunk = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, log_sum), 15));
    // Fold the common factor in now if this chunk's decay would take it below 2^-96; otherwise the corrections
    // are divided by the new factor instead, which multiplies them by at most 2^96.
    const float c_next = c_log + log_chunk;
    const bool fold = c_next < -96.f;
    const float end_base = fold ? log_chunk : -c_log;
    float g_start[4], g_end[4], beta_t[4], ratio[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float lt = __shfl(log_sum, 4 * g + j);
      g_start[j] = pow2(lt + c_log);      // g(t,-1) times the common factor: applies to products with the registers' state
      g_end[j] = pow2(end_base - lt);     // g(15,t) over the factor the registers carry after this chunk
      ratio[j] = pow2(fminf(lt - log_sum, 0.f));  // g(t,n) for t = 4g+j >= n (unused otherwise)
      beta_t[j] = __shfl(cur.beta, 4 * g + j);
    }
    f32x4 a_col, m_col;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int t = 4 * g + j;
      a_col[j] = n < t ? beta_t[j] * ratio[j] * kk[j] : 0.f;
      m_col[j] = n <= t ? ratio[j] * qk[j] : 0.f;
    }
    const DiagBlock dia = publish_system(a_col, m_col, a_off, m_low, a_dia, n, g);

    // Right-hand sides and the state's share of the read-out.
    f32x4 rhs[2], o[2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      rhs[0][j] = beta_t[j] * (bf16_lo(cur.v[j]) - g_start[j] * u[0][j]);
      rhs[1][j] = beta_t[j] * (bf16_hi(cur.v[j]) - g_start[j] * u[1][j]);
      o[0][j] = g_start[j] * w[0][j];
      o[1][j] = g_start[j] * w[1][j];
    }

    if (more) fetch_lane(cur, at, offs, lim_next, g, n);

    // Forward substitution by 4-row groups (rhs turns into delta in place), then the read-out.
    solve_rows(rhs, a_off, dia, n, g);
    readout_rows(o, rhs, m_low, n, g);

    // Token 4g+j's output row is a scalar base of its own, the lane offset the same for all four.
    if (whole) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f32x2 y = {p.scale * o[0][j], p.scale * o[1][j]};
        asm volatile("" : "+v"(out_off));
        *reinterpret_cast<f32x2*>(reinterpret_cast<unsigned char*>(out_at + j * p.H * kD) + out_off) = y;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (4 * g + j <= lim) {
          const f32x2 y = {p.scale * o[0][j], p.scale * o[1][j]};
          asm volatile("" : "+v"(out_off));
          *reinterpret_cast<f32x2*>(reinterpret_cast<unsigned char*>(out_at + j * p.H * kD) + out_off) = y;
        }
      }
    }
    out_at += kC * p.H * kD;

    // The stored state ends inside this chunk (a verify pass whose later tokens may be rejected): the same
    // update with the decay taken up to token n_keep-1 and the later tokens left out, written straight to memory.
    if (n_keep > 0 && n_keep < kC && n_commit < p.T) {
      uint32_t keep_off = lane_off;
      asm volatile("" : "+v"(keep_off));
      const float log_keep = __shfl(log_sum, n_keep - 1);
      const float g_keep = exp2f(log_keep + c_log);
      Split4x2 dk2[2];
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        f32x4 x;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float lt = __shfl(log_sum, 4 * g + j);
          x[j] = 4 * g + j < n_keep ? exp2f(log_keep - lt) * rhs[c][j] : 0.f;
        }
        dk2[c] = split2(x);
      }
#pragma unroll
      for (int rt = 0; rt < 8; ++rt) {
        const u32x2 kt = *reinterpret_cast<const u32x2*>(k_chn + chn_row(n) + 8 * g + rt * kChRowTile);
        f32x4 acc[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          acc[c] = S[rt][c];
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[c][j] *= g_keep;
          acc[c] = mfma_two_terms(kt, dk2[c], acc[c]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const f32x2 x = {acc[0][j], acc[1][j]};
          __builtin_nontemporal_store(x, reinterpret_cast<f32x2*>(sout + (keep_off + (16 * rt + j) * kD)));
        }
      }
    }

    // S <- g(15,-1) S + K^T (g(15,t) delta_t), the decay going into the common factor: rows of the B operand are tokens.
    if (fold) {
      const float f = exp2f(c_next);
#pragma unroll
      for (int rt = 0; rt < 8; ++rt)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int j = 0; j < 4; ++j) S[rt][c][j] *= f;
      c_log = 0.f;
    } else {
      c_log = c_next;
    }
    Split4x2 ds[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      f32x4 x;
#pragma unroll
      for (int j = 0; j < 4; ++j) x[j] = g_end[j] * rhs[c][j];
      ds[c] = split2(x);
    }
    const unsigned char* const k_lane = k_chn + chn_row(n) + 8 * g;
#pragma unroll
    for (int rt = 0; rt < 8; ++rt) {
      const u32x2 kt = *reinterpret_cast<const u32x2*>(k_lane + rt * kChRowTile);
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        S[rt][c] = mfma_two_terms(kt, ds[c], S[rt][c]);
      }
    }
    // The per-wavefront matrices are rewritten in the next chunk only after this chunk's reads (program order).
  }

  if (n_commit == p.T) store_tile(S, sout, lane_off, exp2f(c_log));
}


// ---------------------------------------------------------------------------------------------
// KDA: the gate is a vector over key channels, S_t = (I - beta_t k_t k_t^T) diag(alpha_t) S_{t-1} + beta_t k_t v_t^T.
// With P_t = prod_{m<=t} alpha_m (per channel, from the chunk's first token) the same unrolling gives
//     delta_t = beta_t (v_t - S_0^T (P_t k_t)) - sum_{i<t} beta_t ((P_t k_t).(k_i / P_i)) delta_i
//     o_t     = scale ( S_0^T (P_t q_t) + sum_{i<=t} ((P_t q_t).(k_i / P_i)) delta_i )
//     S_C     = diag(P_C) S_0 + sum_i (P_C / P_i) k_i delta_i^T
// i.e. the GDN scheme with the decay folded into the operands: Khat = P k, Qhat = P q, Ktil = k / P and
// Kend = (P_C / P) k are fp32 and enter the products as two rounded bf16 terms each.
// k / P is the one place where a gate is divided by: P is kept >= 2^-100 by letting a pass cover only as
// many tokens of the chunk as that allows (gates below 2^-100 act as 2^-100, so one token always fits);
// the rest of the chunk follows in further passes over the same staged data.  With gates anywhere near
// those of a trained model a pass is always the whole chunk.
//
// Staging per pass, two barriers: (1) 128 threads, one per key channel, run the product of gates down the
// chunk, write a table of P and the number of tokens their channel allows; barrier; (2) every thread
// scales the 8 channels of the one token whose raw k and q it fetched (coalesced 16-byte loads), splits
// and stores them as MFMA operands, token-major for the A operands of the 16x16x32 products and
// channel-major for K^T Delta; barrier; (3) each wavefront consumes them as in the GDN kernel.
constexpr int kTabRow = kD;                                // floats per token row of the P and 1/P tables
constexpr int kKdaTok = 6 * kC * kTokRowB;                 // Khat, Ktil, Qhat x (hi, lo), token-major
constexpr int kKdaChn = 2 * kChnB;                  // Kend (hi, lo), channel-major
constexpr int kKdaTab = kC * kTabRow * 4;                  // P
constexpr int kKdaMisc = kD * 4 + 16;                      // P at the pass's last token per channel; token limits of 2 wavefronts
constexpr int kKdaLds = kKdaTok + kKdaChn + kKdaTab + kKdaMisc + 4 * kWaveB;
static_assert(kKdaLds <= 64 * 1024, "the KDA chunk kernel must fit the default dynamic LDS limit");
constexpr float kMinGate = 7.888609052e-31f;               // 2^-100

struct KdaRaw {
  u32x4 kst, qst;  // staging: 8 channels of one token of K and of Q
};
struct KdaLane {
  uint32_t v[4];   // this lane's two value columns of tokens 4g .. 4g+3
  float beta;      // of token lane%16
};

// All fetches address a uniform per-chunk base with a 32-bit lane offset (a chunk spans < 4 GiB), the offsets handled
// as in fetch_chunk.  In the call's last, ragged chunk tokens past the end are read from the last valid token, which
// keeps every address in bounds; no pass ever covers them, so what they hold does not matter.
__device__ __forceinline__ void kda_fetch(KdaRaw& raw, KdaLane& f, const ChunkParams& p, ChunkOffsets& offs, size_t row0, int t0, int h,
                                          int hk, int col, int g, int n) {
  const int lim = p.T - 1 - t0;  // last valid token of the chunk
  const size_t kq_base = ((row0 + t0) * p.Hk + hk) * kD;
  const size_t base = ((row0 + t0) * p.H + h);
  if (lim < kC - 1) {
    int lim_here = lim;
    asm volatile("" : "+s"(lim_here));  // what follows depends on this, which keeps it a branch (see fetch_staging)
    offs = chunk_offsets(p, lim_here, col, g, n);
  }
  opaque(offs);
  raw.kst = load_at<u32x4>(p.k + kq_base, offs.kq);
  raw.qst = load_at<u32x4>(p.q + kq_base, offs.kq);
#pragma unroll
  for (int j = 0; j < 4; ++j) f.v[j] = load_at<uint32_t>(p.v + base * kD, offs.v[j]);
  f.beta = load_at<float>(p.beta + base, offs.gate);
}

// The 16 gates of one key channel (thread tid < 128 owns channel tid): one scalar base for the chunk, a lane offset
// that advances by one token row per load (and stops advancing at the call's last token).  Gates are positive, so their
// order as floats is their order as unsigned integers; that maximum is one instruction where fmaxf is two (it first
// quiets a signalling NaN).
__device__ __forceinline__ void kda_fetch_gates(float (&al)[kC], const ChunkParams& p, size_t row0, int t0, int h, int chn) {
  const int lim = p.T - 1 - t0;
  const float* const base = p.alpha + ((row0 + t0) * p.H + h) * kD;
  const uint32_t stride = static_cast<uint32_t>(p.H * kD) * 4u;
  uint32_t off = static_cast<uint32_t>(chn) * 4u;
#pragma unroll
  for (int t = 0; t < kC; ++t) {
    asm volatile("" : "+v"(off));
    const uint32_t x = load_at<uint32_t>(base, off);
    al[t] = __builtin_bit_cast(float, max(x, __builtin_bit_cast(uint32_t, kMinGate)));
    off += t < lim ? stride : 0u;
  }
}

__global__ __launch_bounds__(256, 2) void kda_chunk_kernel(ChunkParams p) {
  extern __shared__ __align__(16) unsigned char lds[];
  // Every index here is the same for the whole workgroup; saying so keeps every base address in scalar registers
  // (the divisions run on the vector unit and their results stay in vector registers, and everything computed
  // from them with them, unless they are moved across by hand).
  const int r = to_scalar(blockIdx.x / p.H);
  const int h = blockIdx.x - r * p.H;
  const int b = __builtin_amdgcn_readfirstlane(p.req_idx ? p.req_idx[r] : r);
  const int slot = __builtin_amdgcn_readfirstlane(p.slot_idx ? p.slot_idx[b] : b);
  const int n_commit = __builtin_amdgcn_readfirstlane(p.n_commit_rows ? min(max(p.n_commit_rows[b], 0), p.T) : p.n_commit);
  const int hk = to_scalar(h / (p.H / p.Hk));
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int n = lane & 15, g = lane >> 4;
  const int col = wave * 32 + 2 * n;
  const size_t row0 = static_cast<size_t>(b) * p.T;
  const int chn = tid & (kD - 1);

  // Token-major operand arrays in the order Khat hi, Khat lo, Ktil hi, Ktil lo, Qhat hi, Qhat lo.
  unsigned char* const tok_arr = lds;
  unsigned char* const kend_hi = lds + kKdaTok;
  unsigned char* const kend_lo = kend_hi + kChnB;
  float* const p_tab = reinterpret_cast<float*>(lds + kKdaTok + kKdaChn);   // [16][128] P_t per channel
  float* const p_end = p_tab + kC * kTabRow;                               // [128] P at the last token of the pass
  int* const limit = reinterpret_cast<int*>(p_end + kD);                    // [2] first token the channels of a wavefront refuse
  float* const wave_mat = reinterpret_cast<float*>(lds + kKdaTok + kKdaChn + kKdaTab + kKdaMisc + wave * kWaveB);
  float* const a_off = wave_mat;
  float* const m_low = wave_mat + kC * kMatRow;
  float* const a_dia = wave_mat + 2 * kC * kMatRow;

  const size_t tile = (static_cast<size_t>(slot) * p.H + h) * (kD * kD);
  const float* const sin = p.state_in + tile;
  float* const sout = p.state_out + tile;
  const uint32_t lane_off = static_cast<uint32_t>(4 * g * kD + col);

  // raw and gates are needed only while a pass is being staged, so the next chunk's are fetched into
  // the same registers as soon as the chunk's last pass has been staged.
  KdaRaw raw;
  KdaLane cur, nxt;
  float gates[kC];
  // Kept in registers for the whole call (the empty asm stops the compiler from recomputing them per chunk).
  ChunkOffsets offs = chunk_offsets(p, kC - 1, col, g, n);
  opaque(offs);
  kda_fetch(raw, cur, p, offs, row0, 0, h, hk, col, g, n);
  if (tid < kD) kda_fetch_gates(gates, p, row0, 0, h, chn);
  f32x4 S[8][2];
#pragma unroll
  for (int rt = 0; rt < 8; ++rt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const f32x2 x = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(sin + (lane_off + (16 * rt + j) * kD)));
      S[rt][0][j] = x[0];
      S[rt][1][j] = x[1];
    }
  __builtin_amdgcn_sched_barrier(0);

  if (n_commit == 0 && sout != sin) store_tile(S, sout, lane_off);
  const int n_chunks = (p.T + kC - 1) / kC;
  for (int ch = 0; ch < n_chunks; ++ch) {
    const int t0 = ch * kC;
    const int n_tok = min(kC, p.T - t0);
    int first = 0;  // the pass covers tokens [first, stop) of the chunk
    while (first < n_tok) {
      // (1) Per channel: running product of gates from `first`, and where it would drop below 2^-100.
      if (tid < kD) {
        // The product keeps running past the token where it leaves the range; those entries are never used.
        float prod = 1.f;
        int mine = n_tok;  // the first token that some channel of this wavefront refuses: a scalar, from wave-wide votes
#pragma unroll
        for (int t = 0; t < kC; ++t) {
          prod *= t >= first ? gates[t] : 1.f;
          if (t > 0 && __builtin_amdgcn_ballot_w64(prod < kMinGate && t > first) != 0) mine = min(mine, t);
          p_tab[t * kTabRow + chn] = prod;
        }
        if (lane == 0) limit[wave] = mine;
      }
      __syncthreads();  // also: every wavefront has finished consuming the previous pass
      int stop = __builtin_amdgcn_readfirstlane(min(limit[0], limit[1]));  // the same for all lanes
      // A pass never straddles the token after which the state is stored: that state is then simply the tile
      // as it stands after the pass.
      const int n_keep = n_commit - t0;
      if (first < n_keep && n_keep < stop) stop = n_keep;

      // (2) Operands of this pass from the raw token this thread fetched.
      {
        const int tok = tid >> 4, c8 = (tid & 15) * 8;
        const bool live = tok >= first && tok < stop;
        const f32x4 pa = *reinterpret_cast<const f32x4*>(p_tab + tok * kTabRow + c8),
                    pb = *reinterpret_cast<const f32x4*>(p_tab + tok * kTabRow + c8 + 4);
        const f32x4 ea = *reinterpret_cast<const f32x4*>(p_tab + (stop - 1) * kTabRow + c8),
                    eb = *reinterpret_cast<const f32x4*>(p_tab + (stop - 1) * kTabRow + c8 + 4);
        if (tok == 0) {
          *reinterpret_cast<f32x4*>(p_end + c8) = ea;
          *reinterpret_cast<f32x4*>(p_end + c8 + 4) = eb;
        }
        float khat[8], ktil[8], qhat[8], kend[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t kw = raw.kst[e >> 1], qw = raw.qst[e >> 1];
          const float kf = (e & 1) ? bf16_hi(kw) : bf16_lo(kw), qf = (e & 1) ? bf16_hi(qw) : bf16_lo(qw);
          const float pt = e < 4 ? pa[e & 3] : pb[e & 3], pe = e < 4 ? ea[e & 3] : eb[e & 3];
          const float it = __builtin_amdgcn_rcpf(pt);  // garbage for a token outside the pass, which `live` discards
          khat[e] = live ? kf * pt : 0.f;
          ktil[e] = live ? kf * it : 0.f;
          qhat[e] = live ? qf * pt : 0.f;
          kend[e] = live ? kf * (pe * it) : 0.f;
        }
        const float* const src[3] = {khat, ktil, qhat};
#pragma unroll
        for (int a = 0; a < 3; ++a) {
          const Split4x2 x = split2(f32x4{src[a][0], src[a][1], src[a][2], src[a][3]}),
                         y = split2(f32x4{src[a][4], src[a][5], src[a][6], src[a][7]});
          unsigned char* const dst = tok_arr + (2 * a) * kC * kTokRowB + tok * kTokRowB + c8 * 2;
          *reinterpret_cast<u32x4*>(dst) = u32x4{x.hi[0], x.hi[1], y.hi[0], y.hi[1]};
          *reinterpret_cast<u32x4*>(dst + kC * kTokRowB) = u32x4{x.lo[0], x.lo[1], y.lo[0], y.lo[1]};
        }
        {
          const Split4x2 x = split2(f32x4{kend[0], kend[1], kend[2], kend[3]}), y = split2(f32x4{kend[4], kend[5], kend[6], kend[7]});
          const uint32_t hi[4] = {x.hi[0], x.hi[1], y.hi[0], y.hi[1]}, lo[4] = {x.lo[0], x.lo[1], y.lo[0], y.lo[1]};
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int at = chn_row(c8 + e) + tok * 2;
            *reinterpret_cast<uint16_t*>(kend_hi + at) = static_cast<uint16_t>((e & 1) ? (hi[e >> 1] >> 16) : (hi[e >> 1] & 0xffffu));
            *reinterpret_cast<uint16_t*>(kend_lo + at) = static_cast<uint16_t>((e & 1) ? (lo[e >> 1] >> 16) : (lo[e >> 1] & 0xffffu));
          }
        }
      }
      __syncthreads();
      // (3) Gram matrices and Khat S_0, Qhat S_0 (three leading cross products of the two-term operands).
      f32x4 kk = {0.f, 0.f, 0.f, 0.f}, qk = {0.f, 0.f, 0.f, 0.f};
      f32x4 u[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}, w[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int off = n * kTokRowB + (32 * s + 4 * g) * 2;
        bf16x8 f[6];
#pragma unroll
        for (int a = 0; a < 6; ++a) {
          const unsigned char* const src = tok_arr + a * kC * kTokRowB + off;
          f[a] = join8(*reinterpret_cast<const u32x2*>(src), *reinterpret_cast<const u32x2*>(src + 32));
        }
        // f: Khat hi, Khat lo, Ktil hi, Ktil lo, Qhat hi, Qhat lo
        kk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[1], f[2], kk, 0, 0, 0);
        kk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[0], f[3], kk, 0, 0, 0);
        kk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[0], f[2], kk, 0, 0, 0);
        qk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[5], f[2], qk, 0, 0, 0);
        qk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[4], f[3], qk, 0, 0, 0);
        qk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[4], f[2], qk, 0, 0, 0);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const Split4x2 lo_tile = split2(S[2 * s][c]), hi_tile = split2(S[2 * s + 1][c]);
          const bf16x8 b_hi = join8(lo_tile.hi, hi_tile.hi), b_lo = join8(lo_tile.lo, hi_tile.lo);
          u[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[1], b_hi, u[c], 0, 0, 0);
          w[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[5], b_hi, w[c], 0, 0, 0);
          u[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[0], b_lo, u[c], 0, 0, 0);
          w[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[4], b_lo, w[c], 0, 0, 0);
          u[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[0], b_hi, u[c], 0, 0, 0);
          w[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[4], b_hi, w[c], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);  // keeps the next slice's 6 fragments and splits out of this one's registers
      }

      float beta_t[4];
      f32x4 a_col, m_col;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int t = 4 * g + j;
        const float bt = __shfl(cur.beta, t);
        beta_t[j] = (t >= first && t < stop) ? bt : 0.f;
        a_col[j] = n < t ? beta_t[j] * kk[j] : 0.f;
        m_col[j] = n <= t ? qk[j] : 0.f;
      }
      const DiagBlock dia = publish_system(a_col, m_col, a_off, m_low, a_dia, n, g);

      // The next chunk's inputs are requested here, after the register-hungry products above.
      __builtin_amdgcn_sched_barrier(0);
      if (stop == n_tok && ch + 1 < n_chunks) {
        // An opaque copy of the next chunk's first token: otherwise the addresses below are formed at the top
        // of the chunk as 64-bit vector pointers, one per load, and live (or spill) through all of it.
        int t_next = t0 + kC;
        asm volatile("" : "+s"(t_next));
        kda_fetch(raw, nxt, p, offs, row0, t_next, h, hk, col, g, n);
        if (tid < kD) kda_fetch_gates(gates, p, row0, t_next, h, chn);
      }
      __builtin_amdgcn_sched_barrier(0);

      f32x4 rhs[2], o[2];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        rhs[0][j] = beta_t[j] * (bf16_lo(cur.v[j]) - u[0][j]);
        rhs[1][j] = beta_t[j] * (bf16_hi(cur.v[j]) - u[1][j]);
      }
      o[0] = w[0];
      o[1] = w[1];
      solve_rows(rhs, a_off, dia, n, g);
      readout_rows(o, rhs, m_low, n, g);

#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int t = 4 * g + j;
        if (t >= first && t < stop) {
          const f32x2 y = {p.scale * o[0][j], p.scale * o[1][j]};
          *reinterpret_cast<f32x2*>(p.out + ((row0 + t0 + t) * p.H + h) * kD + col) = y;
        }
      }

      // S <- diag(P_end) S + Kend^T Delta.
      Split4x2 ds[2] = {split2(rhs[0]), split2(rhs[1])};
      const int k_lane = chn_row(n) + 8 * g;
#pragma unroll
      for (int rt = 0; rt < 8; ++rt) {
        const int at = k_lane + rt * kChRowTile;
        const u32x2 e_hi = *reinterpret_cast<const u32x2*>(kend_hi + at);
        const s16x4 e_lo = __builtin_bit_cast(s16x4, *reinterpret_cast<const u32x2*>(kend_lo + at));
        const f32x4 row_scale = *reinterpret_cast<const f32x4*>(p_end + 16 * rt + 4 * g);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          f32x4 acc = S[rt][c];
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[j] *= row_scale[j];
          acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(e_lo, __builtin_bit_cast(s16x4, ds[c].hi), acc, 0, 0, 0);
          S[rt][c] = mfma_two_terms(e_hi, ds[c], acc);
        }
      }
      first = stop;
      if (t0 + first == n_commit && n_commit < p.T) store_tile(S, sout, lane_off);  // first > 0 here
    }
    cur = nxt;
  }

  if (n_commit == p.T) store_tile(S, sout, lane_off);
}

}  // namespace

namespace {

template <bool KDA>
sa_status chunk_launch(bool dry_run, const char* name, const void* q, const void* k, const void* v, const float* alpha,
                       const float* beta, const float* state_in, float* state_out, float* out, const int32_t* slot_idx,
                       const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv, float scale, int n_commit,
                       const int32_t* n_commit_rows, void* stream) {
  SA_REQUIRE(B >= 0 && T >= 1, SA_EINVAL, "%s: need B >= 0 and T >= 1 (B=%d, T=%d)", name, B, T);
  SA_REQUIRE(H >= 1 && Hk >= 1 && H % Hk == 0, SA_EINVAL, "%s: H must be a positive multiple of Hk (H=%d, Hk=%d)", name, H, Hk);
  SA_REQUIRE(n_commit >= 0 && n_commit <= T, SA_EINVAL, "%s: n_commit=%d outside [0,T=%d]", name, n_commit, T);
  SA_REQUIRE(dk == kD && dv == kD, SA_EUNSUPPORTED, "%s: (dk,dv)=(%d,%d), only (128,128) is supported", name, dk, dv);
  const int rows = req_idx ? n_req : B;
  SA_REQUIRE(rows >= 0 && rows <= B, SA_EINVAL, "%s: n_req=%d outside [0,B=%d]", name, n_req, B);
  if (rows == 0) return SA_OK;
  SA_REQUIRE(q && k && v && alpha && beta && state_in && state_out && out, SA_EINVAL, "%s: null pointer", name);
  SA_REQUIRE(sa::aligned(q, 16) && sa::aligned(k, 16) && sa::aligned(v, 16) && sa::aligned(state_in, 16) &&
                 sa::aligned(state_out, 16) && sa::aligned(out, 16) && sa::aligned(alpha, KDA ? 16 : 4) && sa::aligned(beta, 4) &&
                 sa::aligned(slot_idx, 4) && sa::aligned(req_idx, 4) && sa::aligned(n_commit_rows, 4),
             SA_EINVAL, "%s: misaligned pointer", name);
  SA_REQUIRE(static_cast<long long>(rows) * H <= 0x7fffffffLL, SA_EUNSUPPORTED, "%s: too many tiles", name);
  if (dry_run) return SA_OK;

  ChunkParams p{static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v),
                alpha, beta, state_in, state_out, out, slot_idx, req_idx, T, H, Hk, scale, n_commit, n_commit_rows};
  const dim3 grid(static_cast<unsigned>(rows * H));
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (KDA) {
    sa::launch(SA_K_KDA_CHUNK, kda_chunk_kernel, grid, dim3(256), kKdaLds, s, p);
  } else {
    if (T <= kC)
      sa::launch(SA_K_GDN_CHUNK, gdn_chunk_kernel<true>, grid, dim3(256), kStageB + 4 * kWaveB, s, p);
    else
      sa::launch(SA_K_GDN_CHUNK, gdn_chunk_kernel<false>, grid, dim3(256), 2 * kStageB + 4 * kWaveB, s, p);
  }
  return sa::check_launch(name);
}

}  // namespace

// The chunk-parallel kernels under the names and rules of the decode steps (used by them for longer calls).
sa_status sa::chunked_steps(bool kda, bool dry_run, const char* name, const void* q, const void* k, const void* v,
                            const float* alpha, const float* beta, const float* state_in, float* state_out, float* out,
                            const int32_t* slot_idx, const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv,
                            float scale, int n_commit, const int32_t* n_commit_rows, void* stream) {
  if (kda)
    return chunk_launch<true>(dry_run, name, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk,
                              dk, dv, scale, n_commit, n_commit_rows, stream);
  return chunk_launch<false>(dry_run, name, q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B, T, H, Hk,
                             dk, dv, scale, n_commit, n_commit_rows, stream);
}

extern "C" sa_status gdn_chunk_steps(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                                     const float* state_in, float* state_out, float* out, const int32_t* slot_idx,
                                     const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv,
                                     float scale, int n_commit, void* stream) {
  return chunk_launch<false>(false, "gdn_chunk_steps", q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B,
                             T, H, Hk, dk, dv, scale, n_commit, nullptr, stream);
}

extern "C" sa_status kda_chunk_steps(const void* q, const void* k, const void* v, const float* alpha, const float* beta,
                                     const float* state_in, float* state_out, float* out, const int32_t* slot_idx,
                                     const int32_t* req_idx, int n_req, int B, int T, int H, int Hk, int dk, int dv,
                                     float scale, int n_commit, void* stream) {
  return chunk_launch<true>(false, "kda_chunk_steps", q, k, v, alpha, beta, state_in, state_out, out, slot_idx, req_idx, n_req, B,
                            T, H, Hk, dk, dv, scale, n_commit, nullptr, stream);
}
