// Device side of the paged GQA decode attention (split kernel body, merge body), shared by the stand-alone
// kernels of attn_decode.hip and the fused per-layer kernel of layer_fused.hip.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "samixers.h"

namespace sa {

// Arguments of one attention launch (split and merge).
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

// One prepared attention call: rows = request rows to launch over (0: nothing to do).
struct AttnLaunch {
  AttnParams p;
  int rows;
};

// Argument checks of attn_decode; on success with `launch` not null, fills it (defined in attn_decode.hip).
sa_status attn_prepare(const void* q, const void* kpool, const void* vpool, int n_pages, const int32_t* page_table, int max_pages,
                 const int32_t* seq_lens, const int32_t* req_idx, int n_req, float* out, int B, int T, int Hq, int Hkv, int D,
                 int page_size, int max_seq_len, int window, float scale, void* workspace, size_t workspace_bytes,
                 AttnLaunch* launch);

}  // namespace sa

namespace {

using sa::AttnParams;

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
// The work of one workgroup (256 threads) for KV head g, page range `split` of row r of the request list.
struct AttnShared {
  float o[kWaves][16][kD];
  float m[kWaves][16];
  float l[kWaves][16];
};


template <int NT>
__device__ __forceinline__ void attn_split_body(const AttnParams& p, const int g, const int split, const int r, AttnShared& sm) {
  float (&sm_o)[kWaves][16][kD] = sm.o;
  float (&sm_m)[kWaves][16] = sm.m;
  float (&sm_l)[kWaves][16] = sm.l;
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
  // The page ranges are cut from the sequence's own length (known only here), so that all ranges of a (request, KV head)
  // carry the same work and a short sequence becomes several short ranges instead of one long and some empty ones;
  // the host's pages_per_split, planned from the longest possible sequence, is the upper limit.
  const int own = (((page_end - page_first + p.nsplit - 1) / p.nsplit) + kWaves - 1) / kWaves * kWaves;
  const int per_split = min(max(own, kWaves), p.pages_per_split);
  const int ps = page_first + split * per_split;
  const int pe = min(page_end, ps + per_split);

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
    // The pages of the range are visited cyclically from a starting point that differs from workgroup to workgroup
    // (the running softmax does not care about the order).  Workgroups start together and advance at the same pace;
    // with a regular page table (pages of a request in a row, requests at a fixed distance) they would otherwise all
    // be reading addresses a fixed multiple of the range length apart at any moment, which a few memory channels serve.
    const uint32_t mix = static_cast<uint32_t>(r * p.nsplit + split) * 0x9E3779B1u;
    const int rot = static_cast<int>((mix >> 8) % static_cast<uint32_t>(n_iter));
    auto page_of = [&](int it) {
      int pos = it + rot;
      pos -= pos >= n_iter ? n_iter : 0;
      return first + pos * kWaves;
    };
    // Lane i of the wavefront keeps the physical page of iteration (64*c + i).
    auto load_table = [&](int base_iter) {
      const int it = base_iter + lane;
      const int pg = it < n_iter ? page_of(it) : pe;
      int e = pg < pe ? table[pg] : 0;
      return min(max(e, 0), p.n_pages - 1);
    };
    int tbl = load_table(0);
    PageFrags cur, nxt;
    load_page(cur, p.kpool, p.vpool, __builtin_amdgcn_readlane(tbl, 0), p.Hkv, g, lane);

    for (int it = 0; it < n_iter; ++it) {
      const int pg = page_of(it);
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
        // Both terms of P in one 16x16x32 product: its contraction index runs over (token, term), slots 0-3 of a
        // lane's 8 holding tokens 4*grp..+3 with the first term and slots 4-7 the same tokens with the second, so
        // the V operand is the lane's 4 values twice.
        const bf16x8 p_two = __builtin_bit_cast(bf16x8, uint4{hi.x, hi.y, lo.x, lo.y});

#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
          f32x4 acc = o[n][nb];
          acc[0] *= corr;
          acc[1] *= corr;
          acc[2] *= corr;
          acc[3] *= corr;
          const bf16x8 v_twice = __builtin_bit_cast(bf16x8, uint4{cur.v[nb].x, cur.v[nb].y, cur.v[nb].x, cur.v[nb].y});
          o[n][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v_twice, p_two, acc, 0, 0, 0);
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

// One thread per output element of a (request, KV head, query row): combine the nsplit partials in index
// order and normalise.  The partials are fetched eight ranges at a time (sixteen independent loads in flight, not
// one after the other) and folded into a running maximum, normaliser and sum by the online-softmax rule.
// `item` = (r * Hkv + g) * R + row; d = the output dimension this thread owns.
__device__ __forceinline__ void attn_merge_body(const AttnParams& p, const int item, const int d) {
  constexpr int kBatch = 8;
  const int row = item % p.R;
  const int g = (item / p.R) % p.Hkv;
  const int r = item / (p.R * p.Hkv);
  const int b = p.req_idx ? p.req_idx[r] : r;
  const size_t part0 = (static_cast<size_t>(r) * p.Hkv + g) * p.nsplit * p.R + row;
  const float2* const ml = p.part_ml + part0;         // range s at ml[s * R]
  const float* const po = p.part_o + part0 * kD + d;  // range s at po[s * R * kD]
  float m = kNegBig, l = 0.f, acc = 0.f;
  for (int s0 = 0; s0 < p.nsplit; s0 += kBatch) {
    float2 mlv[kBatch];
    float ov[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const size_t s = static_cast<size_t>(min(s0 + j, p.nsplit - 1));  // past the end: the last range again, left out below
      mlv[j] = ml[s * p.R];
      ov[j] = po[s * p.R * kD];
    }
    float m_new = m;
#pragma unroll
    for (int j = 0; j < kBatch; ++j)
      if (s0 + j < p.nsplit) m_new = fmaxf(m_new, mlv[j].x);
    const float keep = exp2f(m - m_new);
    l *= keep;
    acc *= keep;
#pragma unroll
    for (int j = 0; j < kBatch; ++j)
      if (s0 + j < p.nsplit) {
        const float f = exp2f(mlv[j].x - m_new);
        l = fmaf(mlv[j].y, f, l);
        acc = fmaf(ov[j], f, acc);
      }
    m = m_new;
  }
  const int t = row / p.G, hq = g * p.G + row % p.G;
  p.out[((static_cast<size_t>(b) * p.T + t) * p.Hq + hq) * kD + d] = l > 0.f ? acc / l : 0.f;
}

}  // namespace
