// Paged GQA decode attention (full and sliding-window) and the KV append kernel, gfx950.
//
// Appendix B of the paper defines FA as grouped-query softmax attention over the whole cache and SWA
// as the same weights restricted to the w most recent positions; its cost law for decode is the
// K/V stream (2 * t * h_kv * d_h * b bytes per layer), so the kernel is built around reading every
// cached K and V byte exactly once, fully coalesced.
//
// Split over pages.  A workgroup handles one (request, KV head, page range); its 4 wavefronts take
// the pages of the range round-robin, each keeping its own running maximum, normaliser and output,
// which are merged through LDS at the end and written as one partial per workgroup.  A second
// kernel merges the partials of all ranges in a fixed order.
//
// Matrix-core mapping.  The Hq/Hkv query heads that share a KV head (times the T new tokens) form up
// to 16 query rows, which is one MFMA N-tile:
//   scores   S^T[token][row] = K[token][:] . Q[row][:]      4 x mfma_f32_16x16x32_bf16 per page
//   output   O^T[dim][row]  += V^T[dim][token] P^T[token][row]   8 x 2 x mfma_f32_16x16x16_bf16
// The in-page K and V layouts (see the header) are exactly the A-operand register layouts of those
// two instructions, so lane l loads its fragment from `block + i*stride + l*width`: no LDS staging,
// no transposes.  S^T leaves the matrix core with lane (row = l%16, group = l/16) holding tokens
// 4*group..4*group+3 of its row, which is also the B-operand layout of the second product, and O^T
// keeps that same row in the lane, so the whole online softmax is lane-local except for a 2-step
// maximum over the 4 token groups.  Probabilities are split into two bf16 terms (p = hi + lo) so the
// second product carries ~16 mantissa bits of p instead of 8.
#include "common.h"

namespace {

constexpr int kPage = 16;
constexpr int kD = 128;
constexpr int kBlockElems = kPage * kD;  // bf16 elements of one (page, head) K or V block
constexpr int kWaves = 4;
constexpr float kNegBig = -1.0e30f;
// Dynamic LDS requested on top of the 32.5 KiB the split kernel uses, so that only 2 workgroups fit
// in a CU's 160 KiB.  With 3 resident workgroups the same kernel streams 2-3 % slower and with 4
// (forced by a register cap) 5-15 % slower: more concurrent page streams than that only add
// contention in the memory system.
constexpr int kOccupancyPadBytes = 24 * 1024;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

struct AttnParams {
  const uint16_t* q;
  const uint16_t* kpool;
  const uint16_t* vpool;
  const int32_t* page_table;
  const int32_t* seq_lens;
  const int32_t* req_idx;
  float* part_o;    // [n_req][Hkv][nsplit][R][D]
  float2* part_ml;  // [n_req][Hkv][nsplit][R]  (running max in log2 units, normaliser)
  float* out;
  int n_pages, max_pages;
  int T, Hq, Hkv, G, R;
  int nsplit, pages_per_split;
  int max_seq_len, window;
  float scale_log2;  // softmax scale times log2(e)
};

struct SplitPlan {
  int nsplit, pages_per_split;
};

// Host-side plan: how many page ranges per (request, KV head) and how long each is.  Only bounds
// known on the host enter (the real lengths live in device memory); ranges past a sequence's end
// exit at once.
SplitPlan plan_splits(int n_req, int Hkv, int T, int max_seq_len, int window) {
  long long max_pages = (static_cast<long long>(max_seq_len) + kPage - 1) / kPage;
  if (window > 0) {
    long long span = (static_cast<long long>(window) + T - 1 + kPage - 1) / kPage + 1;
    if (span < max_pages) max_pages = span;
  }
  if (max_pages < 1) max_pages = 1;
  const long long pairs = static_cast<long long>(n_req) * Hkv;
  auto make = [&](long long ranges) {
    long long per = (max_pages + ranges - 1) / ranges;
    per = (per + kWaves - 1) / kWaves * kWaves;
    SplitPlan sp;
    sp.pages_per_split = static_cast<int>(per);
    sp.nsplit = static_cast<int>((max_pages + per - 1) / per);
    return sp;
  };
  // Cost model.  The K/V stream runs fastest with 2 workgroups per CU (see kOccupancyPadBytes), so a
  // launch of N equal workgroups takes about ceil(N / slots) rounds, slots = 2 * CUs; a workgroup costs
  // its pages plus a start-up (lengths, page ids, first page: three dependent memory latencies, about
  // 8 pages' worth of streaming time).  Pick the range count that minimises rounds * (pages + start-up).
  // Full attention keeps at least 4 ranges when the context allows: real lengths are ragged and only
  // known on the device, and finer ranges even out the load (measured: 978 us against 1060 us for one
  // range at lengths uniform in [8192, 32768]).
  static const long long slots = [] {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess || prop.multiProcessorCount < 1) {
      (void)hipGetLastError();
      return 512LL;
    }
    return 2LL * prop.multiProcessorCount;
  }();
  const long long startup_pages = 8, min_pages = 16;
  long long most = max_pages / min_pages;
  most = most < 1 ? 1 : (most > 64 ? 64 : most);
  long long least = window > 0 ? 1 : 4;
  least = least > most ? most : least;
  long long best = least, best_cost = -1;
  for (long long n = least; n <= most; ++n) {
    const SplitPlan sp = make(n);
    const long long groups = pairs * sp.nsplit;
    const long long cost = ((groups + slots - 1) / slots) * (sp.pages_per_split + startup_pages);
    if (best_cost < 0 || cost < best_cost) {
      best_cost = cost;
      best = n;
    }
  }
  return make(best);
}

// Two floats to a packed bf16 pair (a in the low half), round to nearest even: one v_cvt_pk_bf16_f32.
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

struct PageFrags {
  uint4 k[4];
  uint2 v[8];
};

__device__ __forceinline__ void load_page(PageFrags& f, const uint16_t* kpool, const uint16_t* vpool, int phys, int Hkv,
                                          int g, int lane) {
  const size_t block = (static_cast<size_t>(phys) * Hkv + g) * kBlockElems;
  const uint16_t* kb = kpool + block + lane * 8;
  const uint16_t* vb = vpool + block + lane * 4;
  // every K and V byte is read once per step: non-temporal loads
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb + i * 512));
    f.k[i] = uint4{t[0], t[1], t[2], t[3]};
  }
#pragma unroll
  for (int nb = 0; nb < 8; ++nb) {
    const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(vb + nb * 256));
    f.v[nb] = uint2{t[0], t[1]};
  }
}

// NT = number of 16-row query tiles per KV head (1: up to 16 rows, 2: up to 32, e.g. 8 new tokens x 4 heads).
// K and V fragments are loaded once per page and used for every tile.
// The second launch bound asks the compiler to fit 2 wavefronts per SIMD: the two-tile variant otherwise
// takes 268 registers, runs one workgroup per CU and stalls on every page (2.19 ms against 1.35 ms).
template <int NT>
__global__ __launch_bounds__(256, NT) void attn_split_kernel(AttnParams p) {
  __shared__ float sm_o[kWaves][16][kD];
  __shared__ float sm_m[kWaves][16];
  __shared__ float sm_l[kWaves][16];

  // KV head fastest: consecutive workgroups go to consecutive XCDs, and every KV head carries the
  // same amount of work, whereas page ranges do not (late ranges only exist for long sequences).
  const int g = blockIdx.x, split = blockIdx.y, r = blockIdx.z;
  const int b = p.req_idx ? p.req_idx[r] : r;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int row16 = lane & 15, grp = lane >> 4;

  int L = p.seq_lens[b];
  L = L < p.max_seq_len ? L : p.max_seq_len;
  L = L < 0 ? 0 : L;
  const int lo_first = p.window > 0 ? max(0, L - p.T + 1 - p.window) : 0;
  const int page_first = lo_first / kPage;
  const int page_end = (L + kPage - 1) / kPage;
  const int ps = page_first + split * p.pages_per_split;
  const int pe = min(page_end, ps + p.pages_per_split);

  // This lane's query row in tile n: new token t_row, head g*G + row%G.  Rows >= R are padding (q = 0).
  bool real_row[NT];
  int hi_row[NT], lo_row[NT];
  bf16x8 qf[NT][4];
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    const int row = n * 16 + row16;
    real_row[n] = row < p.R;
    const int t_row = real_row[n] ? row / p.G : p.T - 1;
    hi_row[n] = L - p.T + t_row + 1;
    lo_row[n] = p.window > 0 ? max(0, hi_row[n] - p.window) : 0;
    const uint4 zero = {0u, 0u, 0u, 0u};
    const uint16_t* qp =
        p.q + ((static_cast<size_t>(b) * p.T + t_row) * p.Hq + g * p.G + (real_row[n] ? row % p.G : 0)) * kD + grp * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint4 w = real_row[n] ? *reinterpret_cast<const uint4*>(qp + i * 32) : zero;
      qf[n][i] = __builtin_bit_cast(bf16x8, w);
    }
  }

  float m_run[NT], l_run[NT];
  f32x4 o[NT][8];
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    m_run[n] = kNegBig;
    l_run[n] = 0.f;
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) o[n][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int32_t* table = p.page_table + static_cast<size_t>(b) * p.max_pages;
  const int first = ps + wave;
  const int n_iter = first < pe ? (pe - first + kWaves - 1) / kWaves : 0;

  if (n_iter > 0) {
    // Lane i of the wavefront keeps the physical page of iteration (64*c + i).
    auto load_table = [&](int base_iter) {
      int pg = first + (base_iter + lane) * kWaves;
      int e = pg < pe ? table[pg] : 0;
      return min(max(e, 0), p.n_pages - 1);
    };
    int tbl = load_table(0);
    PageFrags cur, nxt;
    load_page(cur, p.kpool, p.vpool, __builtin_amdgcn_readlane(tbl, 0), p.Hkv, g, lane);

    for (int it = 0; it < n_iter; ++it) {
      const int pg = first + it * kWaves;
      if (it + 1 < n_iter) {
        if (((it + 1) & 63) == 0) tbl = load_table(it + 1);
        load_page(nxt, p.kpool, p.vpool, __builtin_amdgcn_readlane(tbl, (it + 1) & 63), p.Hkv, g, lane);
      }

      const int j0 = pg * kPage + grp * 4;
      // Slots of a boundary page that hold no live token may contain anything (NaN included), and
      // 0 * NaN would poison the output: clear their V entries.  K needs no such care because a
      // masked score is replaced, not multiplied.
      if (pg * kPage < lo_first || pg * kPage + kPage > L) {
        uint32_t keep[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int ja = j0 + 2 * h, jb = ja + 1;
          keep[h] = ((ja >= lo_first && ja < L) ? 0x0000ffffu : 0u) | ((jb >= lo_first && jb < L) ? 0xffff0000u : 0u);
        }
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
          cur.v[nb].x &= keep[0];
          cur.v[nb].y &= keep[1];
        }
      }

#pragma unroll
      for (int n = 0; n < NT; ++n) {
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i)
          s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, cur.k[i]), qf[n][i], s, 0, 0, 0);

        bool ok[4];
        float sv[4];
        float m_loc = kNegBig;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          ok[e] = (j0 + e >= lo_row[n]) && (j0 + e < hi_row[n]);
          sv[e] = ok[e] ? s[e] * p.scale_log2 : kNegBig;
          m_loc = fmaxf(m_loc, sv[e]);
        }
        m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 16));
        m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 32));
        const float m_new = fmaxf(m_run[n], m_loc);
        const float corr = exp2f(m_run[n] - m_new);
        m_run[n] = m_new;
        float pv[4];
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          pv[e] = ok[e] ? exp2f(sv[e] - m_new) : 0.f;
          psum += pv[e];
        }
        l_run[n] = fmaf(l_run[n], corr, psum);

        uint2 hi, lo;
        hi.x = pack_bf16_rne(pv[0], pv[1]);
        hi.y = pack_bf16_rne(pv[2], pv[3]);
        lo.x = pack_bf16_rne(pv[0] - __uint_as_float(hi.x << 16), pv[1] - __uint_as_float(hi.x & 0xffff0000u));
        lo.y = pack_bf16_rne(pv[2] - __uint_as_float(hi.y << 16), pv[3] - __uint_as_float(hi.y & 0xffff0000u));
        const s16x4 p_hi = __builtin_bit_cast(s16x4, hi);
        const s16x4 p_lo = __builtin_bit_cast(s16x4, lo);

#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
          f32x4 acc = o[n][nb];
          acc[0] *= corr;
          acc[1] *= corr;
          acc[2] *= corr;
          acc[3] *= corr;
          const s16x4 vf = __builtin_bit_cast(s16x4, cur.v[nb]);
          acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vf, p_hi, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vf, p_lo, acc, 0, 0, 0);
          o[n][nb] = acc;
        }
      }
      cur = nxt;
    }
  }

  // Merge the 4 wavefronts, one query tile at a time through the same LDS buffer.
  const size_t part = ((static_cast<size_t>(r) * p.Hkv + g) * p.nsplit + split) * p.R;
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    float l = l_run[n];                     // per-lane partial over this lane's token group
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (n > 0) __syncthreads();             // the previous tile has been read out
    if (real_row[n]) {
      if (grp == 0) {
        sm_m[wave][row16] = m_run[n];
        sm_l[wave][row16] = l;
      }
#pragma unroll
      for (int nb = 0; nb < 8; ++nb)
        *reinterpret_cast<float4*>(&sm_o[wave][row16][nb * 16 + grp * 4]) =
            float4{o[n][nb][0], o[n][nb][1], o[n][nb][2], o[n][nb][3]};
    }
    __syncthreads();

    const int rows_here = min(16, p.R - n * 16);
    for (int idx = threadIdx.x; idx < rows_here * kD; idx += 256) {
      const int r16 = idx / kD, d = idx - r16 * kD;
      const int rr = n * 16 + r16;
      float m = sm_m[0][r16];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) m = fmaxf(m, sm_m[w][r16]);
      float lsum = 0.f, acc = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float f = exp2f(sm_m[w][r16] - m);
        lsum = fmaf(sm_l[w][r16], f, lsum);
        acc = fmaf(sm_o[w][r16][d], f, acc);
      }
      if (p.nsplit == 1) {
        // The only range of this (request, KV head): finish here, no partials, no merge kernel.
        const int t = rr / p.G, hq = g * p.G + rr % p.G;
        p.out[((static_cast<size_t>(b) * p.T + t) * p.Hq + hq) * kD + d] = lsum > 0.f ? acc / lsum : 0.f;
      } else {
        p.part_o[(part + rr) * kD + d] = acc;
        if (d == 0) p.part_ml[part + rr] = float2{m, lsum};
      }
    }
  }
}

// One block of 128 threads per (request, KV head, query row): combine the nsplit partials in index
// order and normalise.
__global__ __launch_bounds__(128) void attn_merge_kernel(AttnParams p) {
  const int row = blockIdx.x % p.R;
  const int g = (blockIdx.x / p.R) % p.Hkv;
  const int r = blockIdx.x / (p.R * p.Hkv);
  const int b = p.req_idx ? p.req_idx[r] : r;
  const int d = threadIdx.x;
  const size_t part0 = (static_cast<size_t>(r) * p.Hkv + g) * p.nsplit * p.R + row;
  float m = kNegBig;
  for (int s = 0; s < p.nsplit; ++s) m = fmaxf(m, p.part_ml[part0 + static_cast<size_t>(s) * p.R].x);
  float l = 0.f, acc = 0.f;
  for (int s = 0; s < p.nsplit; ++s) {
    const float2 ml = p.part_ml[part0 + static_cast<size_t>(s) * p.R];
    const float f = exp2f(ml.x - m);
    l = fmaf(ml.y, f, l);
    acc = fmaf(p.part_o[(part0 + static_cast<size_t>(s) * p.R) * kD + d], f, acc);
  }
  const int t = row / p.G, hq = g * p.G + row % p.G;
  p.out[((static_cast<size_t>(b) * p.T + t) * p.Hq + hq) * kD + d] = l > 0.f ? acc / l : 0.f;
}

struct AppendParams {
  const uint16_t* k_new;
  const uint16_t* v_new;
  uint16_t* kpool;
  uint16_t* vpool;
  const int32_t* page_table;
  const int32_t* positions;
  int n_pages, max_pages, T, Hkv;
};

// One block of 128 threads per (row, new token, KV head); thread d moves element d of K and of V.
__global__ __launch_bounds__(128) void kv_append_kernel(AppendParams p) {
  const int g = blockIdx.x % p.Hkv;
  const int i = (blockIdx.x / p.Hkv) % p.T;
  const int b = blockIdx.x / (p.Hkv * p.T);
  const int d = threadIdx.x;
  const long long pos = static_cast<long long>(p.positions[b]) + i;
  if (pos < 0 || pos >= static_cast<long long>(p.max_pages) * kPage) return;
  const int phys = p.page_table[static_cast<size_t>(b) * p.max_pages + pos / kPage];
  if (phys < 0 || phys >= p.n_pages) return;
  const int j = static_cast<int>(pos % kPage);
  const size_t src = ((static_cast<size_t>(b) * p.T + i) * p.Hkv + g) * kD + d;
  const size_t block = (static_cast<size_t>(phys) * p.Hkv + g) * kBlockElems;
  p.kpool[block + ((d >> 3) * kPage + j) * 8 + (d & 7)] = p.k_new[src];
  p.vpool[block + (((d >> 4) * 4 + (j >> 2)) * 16 + (d & 15)) * 4 + (j & 3)] = p.v_new[src];
}

// A single range per (request, KV head) writes the output directly and needs no partials.
size_t workspace_need(int n_req, int Hkv, int R, const SplitPlan& sp) {
  if (sp.nsplit == 1) return 0;
  size_t parts = static_cast<size_t>(n_req) * Hkv * sp.nsplit * R;
  return parts * kD * sizeof(float) + parts * sizeof(float2);
}

}  // namespace

extern "C" size_t attn_decode_workspace_bytes(int n_req, int T, int Hq, int Hkv, int D, int max_seq_len, int window) {
  if (n_req <= 0 || T < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || D != kD || max_seq_len < 0) return 0;
  const int R = T * (Hq / Hkv);
  return workspace_need(n_req, Hkv, R, plan_splits(n_req, Hkv, T, max_seq_len, window));
}

namespace {

sa_status attn_decode_impl(bool dry_run, const void* q, const void* kpool, const void* vpool, int n_pages,
                           const int32_t* page_table, int max_pages, const int32_t* seq_lens, const int32_t* req_idx,
                           int n_req, float* out, int B, int T, int Hq, int Hkv, int D, int page_size, int max_seq_len,
                           int window, float scale, void* workspace, size_t workspace_bytes, void* stream) {
  const char* name = "attn_decode";
  SA_REQUIRE(B >= 0 && T >= 1, SA_EINVAL, "%s: need B >= 0 and T >= 1 (B=%d, T=%d)", name, B, T);
  SA_REQUIRE(Hq >= 1 && Hkv >= 1 && Hq % Hkv == 0, SA_EINVAL, "%s: Hq must be a positive multiple of Hkv", name);
  SA_REQUIRE(D == kD && page_size == kPage, SA_EUNSUPPORTED, "%s: only D=128 and page_size=16 are built (D=%d, page_size=%d)",
             name, D, page_size);
  const int G = Hq / Hkv, R = T * G;
  SA_REQUIRE(R <= 32, SA_EUNSUPPORTED, "%s: T*(Hq/Hkv)=%d exceeds the 32 query rows (two tiles) per KV head", name, R);
  const int rows = req_idx ? n_req : B;
  SA_REQUIRE(rows >= 0 && rows <= B, SA_EINVAL, "%s: n_req=%d outside [0,B=%d]", name, n_req, B);
  if (rows == 0) return SA_OK;
  SA_REQUIRE(n_pages >= 1 && max_pages >= 1 && max_seq_len >= 0, SA_EINVAL, "%s: n_pages, max_pages must be >= 1", name);
  SA_REQUIRE(static_cast<long long>(max_seq_len) <= static_cast<long long>(max_pages) * kPage, SA_EINVAL,
             "%s: max_seq_len=%d does not fit max_pages=%d", name, max_seq_len, max_pages);
  SA_REQUIRE(q && kpool && vpool && page_table && seq_lens && out, SA_EINVAL, "%s: null pointer", name);
  SA_REQUIRE(sa::aligned(q, 16) && sa::aligned(kpool, 16) && sa::aligned(vpool, 16) && sa::aligned(out, 16) &&
                 sa::aligned(workspace, 16) && sa::aligned(page_table, 4) && sa::aligned(seq_lens, 4) &&
                 sa::aligned(req_idx, 4),
             SA_EINVAL, "%s: misaligned pointer", name);
  const SplitPlan sp = plan_splits(rows, Hkv, T, max_seq_len, window);
  const size_t need = workspace_need(rows, Hkv, R, sp);
  SA_REQUIRE(need == 0 || workspace, SA_EINVAL, "%s: workspace is null", name);
  SA_REQUIRE(workspace_bytes >= need, SA_EWORKSPACE, "%s: workspace has %zu bytes, %zu needed", name, workspace_bytes, need);
  SA_REQUIRE(rows <= 65535 && Hkv <= 65535, SA_EUNSUPPORTED, "%s: more than 65535 rows or KV heads per launch", name);
  if (dry_run) return SA_OK;

  AttnParams p;
  p.q = static_cast<const uint16_t*>(q);
  p.kpool = static_cast<const uint16_t*>(kpool);
  p.vpool = static_cast<const uint16_t*>(vpool);
  p.page_table = page_table;
  p.seq_lens = seq_lens;
  p.req_idx = req_idx;
  const size_t parts = static_cast<size_t>(rows) * Hkv * sp.nsplit * R;
  p.part_o = static_cast<float*>(workspace);
  p.part_ml = reinterpret_cast<float2*>(static_cast<float*>(workspace) + parts * kD);
  p.out = out;
  p.n_pages = n_pages;
  p.max_pages = max_pages;
  p.T = T;
  p.Hq = Hq;
  p.Hkv = Hkv;
  p.G = G;
  p.R = R;
  p.nsplit = sp.nsplit;
  p.pages_per_split = sp.pages_per_split;
  p.max_seq_len = max_seq_len;
  p.window = window > 0 ? window : 0;
  p.scale_log2 = scale * 1.4426950408889634f;

  hipStream_t s = static_cast<hipStream_t>(stream);
  if (R <= 16)
    sa::launch(SA_K_ATTN_SPLIT, attn_split_kernel<1>, dim3(Hkv, sp.nsplit, rows), dim3(256), kOccupancyPadBytes, s, p);
  else
    sa::launch(SA_K_ATTN_SPLIT, attn_split_kernel<2>, dim3(Hkv, sp.nsplit, rows), dim3(256), kOccupancyPadBytes, s, p);
  sa_status st = sa::check_launch("attn_decode (split kernel)");
  if (st != SA_OK || sp.nsplit == 1) return st;
  sa::launch(SA_K_ATTN_MERGE, attn_merge_kernel, dim3(static_cast<unsigned>(rows * Hkv * R)), dim3(128), 0, s, p);
  return sa::check_launch("attn_decode (merge kernel)");
}

}  // namespace

extern "C" sa_status attn_decode(const void* q, const void* kpool, const void* vpool, int n_pages,
                                 const int32_t* page_table, int max_pages, const int32_t* seq_lens,
                                 const int32_t* req_idx, int n_req, float* out, int B, int T, int Hq, int Hkv, int D,
                                 int page_size, int max_seq_len, int window, float scale, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  return attn_decode_impl(false, q, kpool, vpool, n_pages, page_table, max_pages, seq_lens, req_idx, n_req, out, B, T, Hq, Hkv, D,
                          page_size, max_seq_len, window, scale, workspace, workspace_bytes, stream);
}

// Argument check of an attention launch without enqueueing anything.
sa_status sa::check_attn_decode(const void* q, const void* kpool, const void* vpool, int n_pages, const int32_t* page_table,
                                int max_pages, const int32_t* seq_lens, const int32_t* req_idx, int n_req, float* out, int B,
                                int T, int Hq, int Hkv, int D, int page_size, int max_seq_len, int window, void* workspace,
                                size_t workspace_bytes) {
  return attn_decode_impl(true, q, kpool, vpool, n_pages, page_table, max_pages, seq_lens, req_idx, n_req, out, B, T, Hq, Hkv, D,
                          page_size, max_seq_len, window, 1.f, workspace, workspace_bytes, nullptr);
}

extern "C" sa_status kv_append(const void* k_new, const void* v_new, void* kpool, void* vpool, int n_pages,
                               const int32_t* page_table, int max_pages, const int32_t* positions, int B, int T,
                               int Hkv, int D, int page_size, void* stream) {
  const char* name = "kv_append";
  SA_REQUIRE(B >= 0 && T >= 1 && Hkv >= 1, SA_EINVAL, "%s: need B >= 0, T >= 1, Hkv >= 1", name);
  SA_REQUIRE(D == kD && page_size == kPage, SA_EUNSUPPORTED, "%s: only D=128 and page_size=16 are built", name);
  if (B == 0) return SA_OK;
  SA_REQUIRE(n_pages >= 1 && max_pages >= 1, SA_EINVAL, "%s: n_pages, max_pages must be >= 1", name);
  SA_REQUIRE(k_new && v_new && kpool && vpool && page_table && positions, SA_EINVAL, "%s: null pointer", name);
  SA_REQUIRE(sa::aligned(k_new, 2) && sa::aligned(v_new, 2) && sa::aligned(kpool, 16) && sa::aligned(vpool, 16) &&
                 sa::aligned(page_table, 4) && sa::aligned(positions, 4),
             SA_EINVAL, "%s: misaligned pointer", name);
  const long long blocks = static_cast<long long>(B) * T * Hkv;
  SA_REQUIRE(blocks <= 0x7fffffffLL, SA_EUNSUPPORTED, "%s: B*T*Hkv too large for one launch", name);
  AppendParams p{static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new), static_cast<uint16_t*>(kpool),
                 static_cast<uint16_t*>(vpool), page_table, positions, n_pages, max_pages, T, Hkv};
  hipStream_t s = static_cast<hipStream_t>(stream);
  sa::launch(SA_K_KV_APPEND, kv_append_kernel, dim3(static_cast<unsigned>(blocks)), dim3(128), 0, s, p);
  return sa::check_launch(name);
}
