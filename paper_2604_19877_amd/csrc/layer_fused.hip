// One launch for all mixers of a layer of a placement stack (decode, one new token per request), gfx950.
//
// Section 6 of the paper ("Per-request placement switching") dispatches every request of a batch to the
// mixer its placement names for the layer.  With one kernel per mixer a layer costs up to six dependent
// launches (FA ranges, FA merge, SWA ranges, SWA merge, KDA, GDN); each ends with a tail in which the
// chip drains, and at small batches the ~6 us a dependent launch costs is most of the step.  Here the
// workgroups of all four mixers form one grid, in the order FA ranges, SWA ranges, KDA tiles, GDN
// tiles: the long attention ranges start first and the short recurrent tiles fill the slots they
// free, so the read-modify-write of the states meets the K/V stream only at that boundary.  A second
// small launch merges the partial results of both attention kinds (merging inside the first launch, by the
// workgroup that finds all other page ranges finished, was measured: with full fences it doubles the step time,
// with device-scope stores and loads it is no faster at batch 128 and slower at batch 8).  The bodies are the ones of the
// stand-alone kernels (attn_device.h, delta_step_device.h); only the index arithmetic differs.
#include "layer_fused.h"

#include "common.h"

namespace {

struct LayerParams {
  sa::AttnParams fa, swa;
  sa::DeltaParams kda, gdn;
  // prefix sums over the grid: [0, end_fa) FA, [end_fa, end_swa) SWA, [end_swa, end_kda) KDA, the rest GDN
  int end_fa, end_swa, end_kda;
};

__global__ __launch_bounds__(256) void layer_decode_kernel(LayerParams p) {
  __shared__ AttnShared sm;
  const int id = blockIdx.x;
  if (id < p.end_swa) {
    const bool full = id < p.end_fa;
    const sa::AttnParams& a = full ? p.fa : p.swa;
    const int i = full ? id : id - p.end_fa;
    // KV head fastest, then page range, then request: the order of the stand-alone grid
    const int pairs = i / a.Hkv;
    attn_split_body<1>(a, i - pairs * a.Hkv, pairs % a.nsplit, pairs / a.nsplit, sm);
  } else {
    // the recurrent tiles of both mixers as one list, visited as the stand-alone step kernels visit theirs
    const int tile = interleaved_tile(id - p.end_swa, static_cast<int>(gridDim.x) - p.end_swa);
    const int n_kda = p.end_kda - p.end_swa;
    if (tile < n_kda)
      delta_step_body<128, 128, true, false>(p.kda, tile, blockIdx.x);
    else
      delta_step_body<128, 128, false, false>(p.gdn, tile - n_kda, blockIdx.x);
  }
}

// A layer whose only mixers are the two recurrent ones: the same two tile bodies in one grid, without the
// attention body's registers and LDS.
struct RecurrentLayerParams {
  sa::DeltaParams kda, gdn;
  int end_kda;  // [0, end_kda) KDA tiles, the rest GDN tiles
};

__global__ __launch_bounds__(256) void layer_recurrent_kernel(RecurrentLayerParams p) {
  const int id = interleaved_tile(blockIdx.x, gridDim.x);  // as the stand-alone step kernels visit their tiles
  if (id < p.end_kda)
    delta_step_body<128, 128, true, false>(p.kda, id, blockIdx.x);
  else
    delta_step_body<128, 128, false, false>(p.gdn, id - p.end_kda, blockIdx.x);
}

struct MergeParams {
  sa::AttnParams fa, swa;
  int end_fa;  // [0, end_fa) rows of the full-attention call, the rest of the sliding-window call
};

__global__ __launch_bounds__(128) void layer_merge_kernel(MergeParams p) {
  const int id = blockIdx.x;
  if (id < p.end_fa)
    attn_merge_body(p.fa, id, threadIdx.x);
  else
    attn_merge_body(p.swa, id - p.end_fa, threadIdx.x);
}

}  // namespace

sa_status sa::layer_fused_launch(const sa::AttnLaunch& fa, const sa::AttnLaunch& swa, const sa::DeltaLaunch& kda,
                                 const sa::DeltaLaunch& gdn, void* stream) {
  const char* name = "placement_decode (fused layer)";
  LayerParams p = {};
  p.fa = fa.p;
  p.swa = swa.p;
  p.kda = kda.p;
  p.gdn = gdn.p;
  const long long n_fa = fa.rows ? static_cast<long long>(fa.rows) * fa.p.Hkv * fa.p.nsplit : 0;
  const long long n_swa = swa.rows ? static_cast<long long>(swa.rows) * swa.p.Hkv * swa.p.nsplit : 0;
  const long long n_kda = kda.rows ? static_cast<long long>(kda.rows) * kda.p.H : 0;
  const long long n_gdn = gdn.rows ? static_cast<long long>(gdn.rows) * gdn.p.H : 0;
  const long long total = n_fa + n_swa + n_kda + n_gdn;
  SA_REQUIRE(total <= 0x7fffffffLL, SA_EUNSUPPORTED, "%s: too many workgroups in one layer", name);
  if (total == 0) return SA_OK;
  SA_REQUIRE((!fa.rows || fa.p.R <= 16) && (!swa.rows || swa.p.R <= 16), SA_EUNSUPPORTED, "%s: more than 16 query rows per KV head",
             name);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (n_fa + n_swa == 0) {
    RecurrentLayerParams rp;
    rp.kda = kda.p;
    rp.gdn = gdn.p;
    rp.end_kda = static_cast<int>(n_kda);
    sa::launch(SA_K_LAYER, layer_recurrent_kernel, dim3(static_cast<unsigned>(total)), dim3(256), 0, s, rp);
    return sa::check_launch(name);
  }
  const long long m_fa = fa.rows && fa.p.nsplit > 1 ? static_cast<long long>(fa.rows) * fa.p.Hkv * fa.p.R : 0;
  const long long m_swa = swa.rows && swa.p.nsplit > 1 ? static_cast<long long>(swa.rows) * swa.p.Hkv * swa.p.R : 0;
  SA_REQUIRE(m_fa + m_swa <= 0x7fffffffLL, SA_EUNSUPPORTED, "%s: too many rows to merge in one layer", name);
  p.end_fa = static_cast<int>(n_fa);
  p.end_swa = static_cast<int>(n_fa + n_swa);
  p.end_kda = static_cast<int>(n_fa + n_swa + n_kda);
  sa::launch(SA_K_LAYER, layer_decode_kernel, dim3(static_cast<unsigned>(total)), dim3(256), kOccupancyPadBytes, s, p);
  sa_status st = sa::check_launch(name);
  if (st != SA_OK || m_fa + m_swa == 0) return st;

  MergeParams m;
  m.fa = fa.p;
  m.swa = swa.p;
  m.end_fa = static_cast<int>(m_fa);
  sa::launch(SA_K_ATTN_MERGE, layer_merge_kernel, dim3(static_cast<unsigned>(m_fa + m_swa)), dim3(128), 0, s, m);
  return sa::check_launch("placement_decode (fused merge)");
}
