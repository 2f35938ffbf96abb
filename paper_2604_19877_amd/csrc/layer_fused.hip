// One launch for all mixers of a layer of a placement stack (decode, one new token per request), gfx950.
//
// Section 6 of the paper ("Per-request placement switching") dispatches every request of a batch to the
// mixer its placement names for the layer.  With one kernel per mixer a layer costs up to six dependent
// launches (FA ranges, FA merge, SWA ranges, SWA merge, KDA, GDN); each ends with a tail in which the
// chip drains, and at small batches the ~6 us a dependent launch costs is most of the step.  Here the
// workgroups of all four mixers form one grid, in the order FA ranges, SWA ranges, KDA tiles, GDN
// tiles: the long attention ranges start first and the short recurrent tiles fill the slots they
// free, so the read-modify-write of the states meets the K/V stream only at that boundary.  The partial
// results of the attention ranges are merged at the head of the NEXT layer's launch (layers write disjoint
// outputs and the stream orders the launches), so a layer costs one launch; only the last fused layer of a
// stack is followed by a small merge launch.  (Merging inside the same launch, by the workgroup that finds all
// other page ranges finished, was measured: with full fences it doubles the step time, with device-scope stores
// and loads it is no faster at batch 128 and slower at batch 8.)  The bodies are the ones of the stand-alone
// kernels (attn_device.h, delta_step_device.h); only the index arithmetic differs.
#include "layer_fused.h"

#include "common.h"

namespace {

// Items of an earlier layer's attention calls to merge: [0, end_fa) of the full-attention call, the rest of the
// sliding-window call; two items (128 threads each) per workgroup of 256.
struct MergeParams {
  sa::AttnParams fa, swa;
  int end_fa, n_items;
};

__device__ __forceinline__ void merge_items(const MergeParams& m, int first_item) {
  const int item = first_item + (threadIdx.x >> 7), d = threadIdx.x & 127;
  if (item >= m.n_items) return;
  if (item < m.end_fa)
    attn_merge_body(m.fa, item, d);
  else
    attn_merge_body(m.swa, item - m.end_fa, d);
}

// Tile `tile` of a layer's recurrent tiles.  One new token per request: one tile body serves both mixers (a kernel that
// carried both took 140 registers instead of 107 and ran three wavefronts per SIMD instead of four), and the tiles are
// visited in the order of `order` (both mixers' requests as one list in request order, a GDN request r stored as ~r):
// state slots are usually handed out in request order, and walking first KDA's requests and then GDN's would visit
// memory in two interleaved passes of 2 MiB runs, which the memory system serves 5 % slower than one pass.
// A verify pass keeps the two bodies (GDN's carries the decay of several steps as a common factor of the tile) and
// the two lists, KDA's first.
template <bool MULTI>
__device__ __forceinline__ void run_tile(const sa::DeltaParams& kda, const sa::DeltaParams& gdn, int tile, int n_kda, float* park,
                                         const int32_t* order, int H) {
  if constexpr (!MULTI) {
    if (order) {
      const int e = tile / H;
      const int entry = order[e];
      const bool is_gdn = entry < 0;
      sa::DeltaParams p = is_gdn ? gdn : kda;
      p.req_idx = nullptr;  // the body then takes the row of the request list as the batch row itself
      delta_step_body<128, 128, true, 0, true>(p, (is_gdn ? ~entry : entry) * H + (tile - e * H), blockIdx.x, park, is_gdn);
      return;
    }
    const bool is_gdn = tile >= n_kda;
    delta_step_body<128, 128, true, 0, true>(is_gdn ? gdn : kda, is_gdn ? tile - n_kda : tile, blockIdx.x, park, is_gdn);
  } else {
    if (tile >= n_kda)
      delta_step_body<128, 128, false, kMaxRegisterSteps128>(gdn, tile - n_kda, blockIdx.x, park);
    else
      delta_step_body<128, 128, true, kMaxRegisterSteps128>(kda, tile, blockIdx.x, park);
  }
}

struct LayerParams {
  MergeParams prev;
  sa::AttnParams fa, swa;
  sa::DeltaParams kda, gdn;
  const int32_t* order;  // see run_tile
  int H;                 // state heads per request (of whichever recurrent launch is not empty)
  // prefix sums over the grid: [0, end_prev) merges of the earlier layer, [end_prev, end_fa) FA, [end_fa, end_swa) SWA,
  // [end_swa, end_kda) KDA, the rest GDN
  int end_prev, end_fa, end_swa, end_kda;
};

// MULTI: the recurrent calls run several tokens or a per-request committed prefix (a verify pass) on the
// register-resident multi-token body; otherwise the one-token body of the decode hot path.
template <bool MULTI>
__global__ __launch_bounds__(256) void layer_decode_kernel(LayerParams p) {
  __shared__ AttnShared sm;
  // one region for whichever tile body this workgroup runs (the KDA body needs the larger one)
  __shared__ __attribute__((aligned(16))) float park[delta_park_floats<128, 128, true, MULTI ? kMaxRegisterSteps128 : 0>()];
  const int id = blockIdx.x;
  if (id < p.end_prev) {
    merge_items(p.prev, 2 * id);
  } else if (id < p.end_swa) {
    const bool full = id < p.end_fa;
    const sa::AttnParams& a = full ? p.fa : p.swa;
    const int i = id - (full ? p.end_prev : p.end_fa);
    // KV head fastest, then page range, then request: the order of the stand-alone grid
    const int pairs = i / a.Hkv;
    attn_split_body<1>(a, i - pairs * a.Hkv, pairs % a.nsplit, pairs / a.nsplit, sm);
  } else {
    // the recurrent tiles of both mixers as one list, visited as the stand-alone step kernels visit theirs
    const int tile = interleaved_tile(id - p.end_swa, static_cast<int>(gridDim.x) - p.end_swa);
    const int n_kda = p.end_kda - p.end_swa;
    run_tile<MULTI>(p.kda, p.gdn, tile, n_kda, park, p.order, p.H);
  }
}

// A layer whose only mixers are the two recurrent ones: the same two tile bodies in one grid, without the
// attention body's registers and LDS.
struct RecurrentLayerParams {
  MergeParams prev;
  sa::DeltaParams kda, gdn;
  const int32_t* order;  // see run_tile
  int H;
  int end_prev, end_kda;  // [0, end_prev) merges of the earlier layer, [end_prev, end_kda) KDA tiles, the rest GDN tiles
};

template <bool MULTI>
__global__ __launch_bounds__(256) void layer_recurrent_kernel(RecurrentLayerParams p) {
  __shared__ __attribute__((aligned(16))) float park[delta_park_floats<128, 128, true, MULTI ? kMaxRegisterSteps128 : 0>()];
  if (static_cast<int>(blockIdx.x) < p.end_prev) {
    merge_items(p.prev, 2 * blockIdx.x);
    return;
  }
  // as the stand-alone step kernels visit their tiles
  const int id = interleaved_tile(static_cast<int>(blockIdx.x) - p.end_prev, static_cast<int>(gridDim.x) - p.end_prev);
  const int n_kda = p.end_kda - p.end_prev;
  run_tile<MULTI>(p.kda, p.gdn, id, n_kda, park, p.order, p.H);
}

__global__ __launch_bounds__(256) void layer_merge_kernel(MergeParams p) { merge_items(p, 2 * blockIdx.x); }

MergeParams merge_params(const sa::PendingMerge& pending) {
  MergeParams m = {};
  m.fa = pending.fa;
  m.swa = pending.swa;
  m.end_fa = pending.n_fa;
  m.n_items = pending.n_fa + pending.n_swa;
  return m;
}

}  // namespace

sa_status sa::layer_fused_launch(const sa::AttnLaunch& fa, const sa::AttnLaunch& swa, const sa::DeltaLaunch& kda,
                                 const sa::DeltaLaunch& gdn, const int32_t* recurrent_order, sa::PendingMerge* pending, void* stream) {
  const char* name = "placement_decode (fused layer)";
  const long long n_fa = fa.rows ? static_cast<long long>(fa.rows) * fa.p.Hkv * fa.p.nsplit : 0;
  const long long n_swa = swa.rows ? static_cast<long long>(swa.rows) * swa.p.Hkv * swa.p.nsplit : 0;
  const long long n_kda = kda.rows ? static_cast<long long>(kda.rows) * kda.p.H : 0;
  const long long n_gdn = gdn.rows ? static_cast<long long>(gdn.rows) * gdn.p.H : 0;
  const MergeParams prev = merge_params(*pending);
  const long long n_prev = (prev.n_items + 1) / 2;
  const long long total = n_prev + n_fa + n_swa + n_kda + n_gdn;
  // what this layer leaves to be merged
  const long long m_fa = fa.rows && fa.p.nsplit > 1 ? static_cast<long long>(fa.rows) * fa.p.Hkv * fa.p.R : 0;
  const long long m_swa = swa.rows && swa.p.nsplit > 1 ? static_cast<long long>(swa.rows) * swa.p.Hkv * swa.p.R : 0;
  SA_REQUIRE(total <= 0x7fffffffLL && m_fa + m_swa <= 0x7ffffffeLL, SA_EUNSUPPORTED, "%s: too many workgroups in one layer", name);
  SA_REQUIRE((!fa.rows || fa.p.R <= 16) && (!swa.rows || swa.p.R <= 16), SA_EUNSUPPORTED, "%s: more than 16 query rows per KV head",
             name);
  if (total == 0) return SA_OK;
  const auto needs_multi = [](const sa::DeltaLaunch& l) { return l.rows && (l.p.T != 1 || l.p.n_commit != 1 || l.p.n_commit_rows); };
  const bool multi = needs_multi(kda) || needs_multi(gdn);
  SA_REQUIRE(!kda.chunked && !gdn.chunked, SA_EUNSUPPORTED, "%s: calls this long run on the chunk-parallel kernels, which are launched on their own", name);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (n_fa + n_swa == 0) {
    RecurrentLayerParams rp = {};
    rp.prev = prev;
    rp.kda = kda.p;
    rp.gdn = gdn.p;
    rp.order = multi ? nullptr : recurrent_order;
    rp.H = kda.rows ? kda.p.H : gdn.p.H;
    rp.end_prev = static_cast<int>(n_prev);
    rp.end_kda = static_cast<int>(n_prev + n_kda);
    if (multi)
      sa::launch(SA_K_LAYER, layer_recurrent_kernel<true>, dim3(static_cast<unsigned>(total)), dim3(256), 0, s, rp);
    else
      sa::launch(SA_K_LAYER, layer_recurrent_kernel<false>, dim3(static_cast<unsigned>(total)), dim3(256), 0, s, rp);
  } else {
    LayerParams p = {};
    p.prev = prev;
    p.fa = fa.p;
    p.swa = swa.p;
    p.kda = kda.p;
    p.gdn = gdn.p;
    p.order = multi ? nullptr : recurrent_order;
    p.H = kda.rows ? kda.p.H : gdn.p.H;
    p.end_prev = static_cast<int>(n_prev);
    p.end_fa = static_cast<int>(n_prev + n_fa);
    p.end_swa = static_cast<int>(n_prev + n_fa + n_swa);
    p.end_kda = static_cast<int>(n_prev + n_fa + n_swa + n_kda);
    // The multi-token tile body parks k, q and gate vectors of up to 4 steps in LDS (30 KiB): with the attention body's
    // 32.5 KiB that already limits a CU to the 2 workgroups the K/V stream wants, so no padding is requested.
    if (multi)
      sa::launch(SA_K_LAYER, layer_decode_kernel<true>, dim3(static_cast<unsigned>(total)), dim3(256), 0, s, p);
    else
      sa::launch(SA_K_LAYER, layer_decode_kernel<false>, dim3(static_cast<unsigned>(total)), dim3(256), kOccupancyPadBytes, s, p);
  }
  const sa_status st = sa::check_launch(name);
  if (st != SA_OK) return st;
  *pending = sa::PendingMerge();
  if (m_fa) pending->fa = fa.p;
  if (m_swa) pending->swa = swa.p;
  pending->n_fa = static_cast<int>(m_fa);
  pending->n_swa = static_cast<int>(m_swa);
  return SA_OK;
}

sa_status sa::layer_merge_flush(sa::PendingMerge* pending, void* stream) {
  const MergeParams m = merge_params(*pending);
  *pending = sa::PendingMerge();
  if (m.n_items == 0) return SA_OK;
  sa::launch(SA_K_ATTN_MERGE, layer_merge_kernel, dim3(static_cast<unsigned>((m.n_items + 1) / 2)), dim3(256), 0,
             static_cast<hipStream_t>(stream), m);
  return sa::check_launch("placement_decode (merge of the last fused layer)");
}
