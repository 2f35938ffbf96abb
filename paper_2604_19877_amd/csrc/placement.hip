// Per-request placement dispatch over a stack of mixer layers (host logic; the fused kernel is in layer_fused.hip).
//
// Section 6 of the paper ("Per-request placement switching") lets every request name a placement,
// i.e. one mixer per layer, and dispatches inside the layer on that name with no global mutable
// state; its scheduler still batches same-placement requests together.  Here a batch may mix
// placements freely: a plan groups the requests per (layer, mixer) once, and every kernel takes
// the group's request list as an indirection.  A step of up to 4 tokens at 128x128 states runs every layer
// as one fused launch, whose head also merges the attention partial results of the layer before; a longer
// step runs the stand-alone kernel of each mixer present.
#include <cstring>
#include <vector>

#include "common.h"
#include "layer_fused.h"

struct sa_plan {
  int L = 0, B = 0;
  // counts[l][m] requests run mixer m at layer l; their ids sit at offset[l][m] of the device list.
  std::vector<int> counts, offsets;
  int32_t* dev_lists = nullptr;  // 2*L*B ints.  First L*B: per layer the requests grouped by mixer (F,S,K,G).  Then L*B: per
                                 // layer the requests of both recurrent mixers as ONE list in request order, a GDN request with
                                 // its sign bit set (~r): the order the fused one-token launch visits the state tiles in.
};

namespace {

int mixer_index(char c) {
  switch (c) {
    case 'F': return 0;
    case 'S': return 1;
    case 'K': return 2;
    case 'G': return 3;
    default: return -1;
  }
}

}  // namespace

extern "C" sa_status placement_plan_create(const char* const* placements, int n_placements, int L,
                                           const int32_t* placement_id, int B, sa_plan** plan_out) {
  const char* name = "placement_plan_create";
  SA_REQUIRE(plan_out, SA_EINVAL, "%s: plan_out is null", name);
  *plan_out = nullptr;
  SA_REQUIRE(placements && n_placements >= 1 && L >= 1 && B >= 0, SA_EINVAL, "%s: bad placement table or sizes", name);
  SA_REQUIRE(B == 0 || placement_id, SA_EINVAL, "%s: placement_id is null", name);
  for (int i = 0; i < n_placements; ++i) {
    SA_REQUIRE(placements[i], SA_EINVAL, "%s: placement %d is null", name, i);
    SA_REQUIRE(static_cast<int>(std::strlen(placements[i])) == L, SA_EINVAL,
               "%s: placement %d has %zu characters, the stack has %d layers", name, i, std::strlen(placements[i]), L);
    for (int l = 0; l < L; ++l)
      SA_REQUIRE(mixer_index(placements[i][l]) >= 0, SA_EINVAL, "%s: placement %d layer %d: unknown mixer '%c'", name,
                 i, l, placements[i][l]);
  }
  for (int r = 0; r < B; ++r)
    SA_REQUIRE(placement_id[r] >= 0 && placement_id[r] < n_placements, SA_EINVAL,
               "%s: request %d names placement %d, only %d exist", name, r, placement_id[r], n_placements);

  sa_plan* plan = new sa_plan;
  plan->L = L;
  plan->B = B;
  plan->counts.assign(static_cast<size_t>(L) * 4, 0);
  plan->offsets.assign(static_cast<size_t>(L) * 4, 0);
  std::vector<int32_t> lists(2 * static_cast<size_t>(L) * B);
  for (int l = 0; l < L; ++l) {
    int at = 0;
    for (int m = 0; m < 4; ++m) {
      plan->offsets[l * 4 + m] = l * B + at;
      for (int r = 0; r < B; ++r)
        if (mixer_index(placements[placement_id[r]][l]) == m) lists[static_cast<size_t>(l) * B + at++] = r;
      plan->counts[l * 4 + m] = l * B + at - plan->offsets[l * 4 + m];
    }
    int32_t* merged = lists.data() + (static_cast<size_t>(L) + l) * B;
    int n = 0;
    for (int r = 0; r < B; ++r) {
      const int m = mixer_index(placements[placement_id[r]][l]);
      if (m == 2) merged[n++] = r;
      if (m == 3) merged[n++] = ~r;
    }
  }
  if (!lists.empty()) {
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&plan->dev_lists), lists.size() * sizeof(int32_t));
    if (e == hipSuccess)
      e = hipMemcpy(plan->dev_lists, lists.data(), lists.size() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      if (plan->dev_lists) (void)hipFree(plan->dev_lists);
      delete plan;
      return sa::fail(SA_EHIP, "%s: %s", name, hipGetErrorString(e));
    }
  }
  *plan_out = plan;
  return SA_OK;
}

extern "C" void placement_plan_destroy(sa_plan* plan) {
  if (!plan) return;
  if (plan->dev_lists) (void)hipFree(plan->dev_lists);
  delete plan;
}

extern "C" int placement_plan_count(const sa_plan* plan, int layer, char mixer) {
  if (!plan || layer < 0 || layer >= plan->L || mixer_index(mixer) < 0) return -1;
  return plan->counts[layer * 4 + mixer_index(mixer)];
}

namespace {

size_t align_up(size_t n, size_t a) { return (n + a - 1) / a * a; }

}  // namespace

// The workspace is two halves used by alternate layers: the partial results of a fused layer are merged by the
// next layer's launch, which writes its own into the other half.  Within a half, full attention's partial results
// sit at the start and the sliding window's behind them (a fused layer launch has both in flight at once).
extern "C" size_t placement_workspace_bytes(const sa_plan* plan, const sa_shapes* sh, int T, int max_seq_len, int window) {
  if (!plan || !sh) return 0;
  size_t need = 0;
  for (int l = 0; l < plan->L; ++l) {
    const int nf = plan->counts[l * 4 + 0], ns = plan->counts[l * 4 + 1];
    const size_t wf = nf ? attn_decode_workspace_bytes(nf, T, sh->Hq, sh->Hkv, sh->D, max_seq_len, 0) : 0;
    const size_t ws = ns ? attn_decode_workspace_bytes(ns, T, sh->Hq, sh->Hkv, sh->D, max_seq_len, window) : 0;
    need = std::max(need, align_up(wf, 256) + ws);
  }
  return 2 * align_up(need, 256);
}

extern "C" sa_status placement_decode(const sa_plan* plan, const sa_layer_io* io, const sa_shapes* sh, int T, int window,
                                      float attn_scale, float rec_scale, void* whole_workspace, size_t whole_workspace_bytes,
                                      void* stream) {
  const char* name = "placement_decode";
  SA_REQUIRE(plan && io && sh, SA_EINVAL, "%s: null plan, io or shapes", name);
  SA_REQUIRE(window > 0, SA_EINVAL, "%s: the sliding window must be positive (window=%d)", name, window);
  SA_REQUIRE(static_cast<long long>(sh->H) * sh->dv == static_cast<long long>(sh->Hq) * sh->D, SA_EINVAL,
             "%s: H*dv must equal Hq*D so that all mixers share the output rows", name);
  const int B = plan->B;
  SA_REQUIRE(sa::aligned(whole_workspace, 256), SA_EINVAL, "%s: the workspace must be aligned to 256 bytes", name);
  const size_t half_bytes = whole_workspace_bytes / 2 / 256 * 256;
  // up to 4 tokens per call: the recurrent mixers stay on the register-resident kernel and the query rows of a KV head fit one tile
  const bool can_fuse = T >= 1 && T <= 4 && sh->dk == 128 && sh->dv == 128 && sh->Hkv >= 1 && T * (sh->Hq / sh->Hkv) <= 16;
  // Two passes over the stack: the first only checks every launch's arguments, so that a bad descriptor
  // anywhere is reported before anything has been enqueued.
  for (int pass = 0; pass < 2; ++pass) {
    const bool check = pass == 0;
    sa::PendingMerge pending;  // partial results of the last fused layer, merged by the next launch
    for (int l = 0; l < plan->L; ++l) {
      const sa_layer_io& x = io[l];
      const int* cnt = &plan->counts[l * 4];
      const int32_t* lists[4];
      for (int m = 0; m < 4; ++m) lists[m] = plan->dev_lists + plan->offsets[l * 4 + m];
      // where each attention kind keeps its partial results: this layer's half of the workspace
      void* const workspace = whole_workspace ? static_cast<char*>(whole_workspace) + (l & 1) * half_bytes : nullptr;
      const size_t workspace_bytes = half_bytes;
      const size_t need_fa = cnt[0] ? attn_decode_workspace_bytes(cnt[0], T, sh->Hq, sh->Hkv, sh->D, x.max_seq_len, 0) : 0;
      const size_t off_swa = std::min(align_up(need_fa, 256), workspace_bytes);
      char* ws_swa = workspace ? static_cast<char*>(workspace) + off_swa : nullptr;
      const size_t ws_swa_bytes = workspace_bytes - off_swa;
      // One fused launch per layer (measured from batch 8 / 2048-token contexts to batch 128 / 16384: 26 % to 0 %
      // faster than one launch per mixer).  A layer with a single mixer present runs the same body as the mixer's
      // stand-alone kernel, but leaves its merge to the next launch (a single sequence through 48 layers: 15-20 %
      // faster per step).
      if (can_fuse) {
        sa::AttnLaunch fa = {}, swa = {};
        sa::DeltaLaunch kda = {}, gdn = {};
        sa_status st = SA_OK;
        if (cnt[0])
          st = sa::attn_prepare(x.q_attn, x.kpool, x.vpool, x.n_pages, x.page_table, x.max_pages, x.seq_lens, lists[0], cnt[0], x.out, B,
                                T, sh->Hq, sh->Hkv, sh->D, sh->page_size, x.max_seq_len, 0, attn_scale, workspace, workspace_bytes,
                                &fa);
        if (st == SA_OK && cnt[1])
          st = sa::attn_prepare(x.q_attn, x.kpool, x.vpool, x.n_pages, x.page_table, x.max_pages, x.seq_lens, lists[1], cnt[1], x.out, B,
                                T, sh->Hq, sh->Hkv, sh->D, sh->page_size, x.max_seq_len, window, attn_scale, ws_swa, ws_swa_bytes,
                                &swa);
        if (st == SA_OK && cnt[2])
          st = sa::delta_prepare(true, x.q, x.k, x.v, x.alpha_vec, x.beta, x.state, x.state, x.out, x.slot_idx, lists[2], cnt[2], B, T,
                                 sh->H, sh->Hk, sh->dk, sh->dv, rec_scale, T, x.n_commit_rows, &kda);
        if (st == SA_OK && cnt[3])
          st = sa::delta_prepare(false, x.q, x.k, x.v, x.alpha_scalar, x.beta, x.state, x.state, x.out, x.slot_idx, lists[3], cnt[3], B,
                                 T, sh->H, sh->Hk, sh->dk, sh->dv, rec_scale, T, x.n_commit_rows, &gdn);
        if (st != SA_OK) return st;
        // The partial results of the layer before are merged into ITS output at the head of this launch, next to this
        // layer's own writes: only safe if the two outputs do not overlap.  If they do (a caller reusing one output
        // buffer for every layer), the merge gets a launch of its own first.
        if (!check && l > 0 && (pending.n_fa || pending.n_swa)) {
          const size_t out_bytes = static_cast<size_t>(B) * T * sh->H * sh->dv * sizeof(float);
          const char* const a = reinterpret_cast<const char*>(io[l - 1].out);
          const char* const b = reinterpret_cast<const char*>(x.out);
          if (a < b + out_bytes && b < a + out_bytes) {
            st = sa::layer_merge_flush(&pending, stream);
            if (st != SA_OK) return st;
          }
        }
        if (!check)
          st = sa::layer_fused_launch(fa, swa, kda, gdn, plan->dev_lists + (static_cast<size_t>(plan->L) + l) * B, &pending, stream);
        if (st != SA_OK) return st;
        continue;
      }
      if (!check) {
        const sa_status st = sa::layer_merge_flush(&pending, stream);
        if (st != SA_OK) return st;
      }

      for (int m = 0; m < 4; ++m) {
        const int n = cnt[m];
        if (n == 0) continue;
        const int32_t* list = lists[m];
        sa_status st;
        if (m == 0 || m == 1) {
          const int w = m == 0 ? 0 : window;
          void* ws = m == 0 ? workspace : ws_swa;
          const size_t ws_bytes = m == 0 ? workspace_bytes : ws_swa_bytes;
          st = check ? sa::check_attn_decode(x.q_attn, x.kpool, x.vpool, x.n_pages, x.page_table, x.max_pages, x.seq_lens, list, n,
                                             x.out, B, T, sh->Hq, sh->Hkv, sh->D, sh->page_size, x.max_seq_len, w, ws, ws_bytes)
                     : attn_decode(x.q_attn, x.kpool, x.vpool, x.n_pages, x.page_table, x.max_pages, x.seq_lens, list, n, x.out, B,
                                   T, sh->Hq, sh->Hkv, sh->D, sh->page_size, x.max_seq_len, w, attn_scale, ws, ws_bytes, stream);
        } else {
          const bool kda = m == 2;
          const float* alpha = kda ? x.alpha_vec : x.alpha_scalar;
          if (check)
            st = sa::delta_prepare(kda, x.q, x.k, x.v, alpha, x.beta, x.state, x.state, x.out, x.slot_idx, list, n, B, T, sh->H,
                                   sh->Hk, sh->dk, sh->dv, rec_scale, T, x.n_commit_rows, nullptr);
          else if (x.n_commit_rows && kda)
            st = kda_decode_step_var(x.q, x.k, x.v, alpha, x.beta, x.state, x.state, x.out, x.slot_idx, list, n, B, T, sh->H,
                                     sh->Hk, sh->dk, sh->dv, rec_scale, x.n_commit_rows, stream);
          else if (x.n_commit_rows)
            st = gdn_decode_step_var(x.q, x.k, x.v, alpha, x.beta, x.state, x.state, x.out, x.slot_idx, list, n, B, T, sh->H,
                                     sh->Hk, sh->dk, sh->dv, rec_scale, x.n_commit_rows, stream);
          else if (kda)
            st = kda_decode_step(x.q, x.k, x.v, alpha, x.beta, x.state, x.state, x.out, x.slot_idx, list, n, B, T, sh->H, sh->Hk,
                                 sh->dk, sh->dv, rec_scale, T, stream);
          else
            st = gdn_decode_step(x.q, x.k, x.v, alpha, x.beta, x.state, x.state, x.out, x.slot_idx, list, n, B, T, sh->H, sh->Hk,
                                 sh->dk, sh->dv, rec_scale, T, stream);
        }
        if (st != SA_OK) return st;
      }
    }
    if (!check) {
      const sa_status st = sa::layer_merge_flush(&pending, stream);
      if (st != SA_OK) return st;
    }
  }
  return SA_OK;
}
