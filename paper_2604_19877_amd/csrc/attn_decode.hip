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
//   output   O^T[dim][row]  += V^T[dim][token] P^T[token][row]   8 x mfma_f32_16x16x32_bf16 (both terms of P at once)
// The in-page K and V layouts (see the header) are exactly the A-operand register layouts of those
// two instructions, so lane l loads its fragment from `block + i*stride + l*width`: no LDS staging,
// no transposes.  S^T leaves the matrix core with lane (row = l%16, group = l/16) holding tokens
// 4*group..4*group+3 of its row, which is also the B-operand layout of the second product, and O^T
// keeps that same row in the lane, so the whole online softmax is lane-local except for a 2-step
// maximum over the 4 token groups.  Probabilities are split into two bf16 terms (p = hi + lo) so the
// second product carries ~16 mantissa bits of p instead of 8; its 32-wide contraction runs over (token, term).
#include <mutex>

#include "attn_device.h"
#include "common.h"

namespace {

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
  // Ranges stay at 16 pages or more.  Shorter ones (down to one page per wavefront, for launches of a few requests
  // with short contexts that fill under half of the slots) were measured on a 48-layer stack of 8 requests x 2048
  // tokens: 0.561 ms per step with this limit, 0.564 ms with 8 pages, 0.570 ms with 4, and a 4-token verify pass
  // 0.727 against 0.815 ms: such a launch lasts as long as its chain of dependent loads (request, length, page
  // ids, first page, and the merge's partial results), which more and shorter ranges do not shorten.
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

// The second launch bound asks the compiler to fit 2 wavefronts per SIMD: the two-tile variant otherwise
// takes 268 registers, runs one workgroup per CU and stalls on every page (2.19 ms against 1.35 ms).
template <int NT>
__global__ __launch_bounds__(256, NT) void attn_split_kernel(AttnParams p) {
  __shared__ AttnShared sm;
  // KV head fastest: consecutive workgroups go to consecutive XCDs, and every KV head carries the
  // same amount of work, whereas page ranges do not (late ranges only exist for long sequences).
  attn_split_body<NT>(p, blockIdx.x, blockIdx.y, blockIdx.z, sm);
}

// One block of 128 threads per (request, KV head, query row).
__global__ __launch_bounds__(128) void attn_merge_kernel(AttnParams p) { attn_merge_body(p, blockIdx.x, threadIdx.x); }

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

// Checks the arguments of one attention call and, when they pass, describes its launches in *launch (if not null).
sa_status sa::attn_prepare(const void* q, const void* kpool, const void* vpool, int n_pages, const int32_t* page_table,
                           int max_pages, const int32_t* seq_lens, const int32_t* req_idx, int n_req, float* out, int B, int T,
                           int Hq, int Hkv, int D, int page_size, int max_seq_len, int window, float scale, void* workspace,
                           size_t workspace_bytes, sa::AttnLaunch* launch) {
  const char* name = "attn_decode";
  if (launch) launch->rows = 0;
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
  SA_REQUIRE(static_cast<long long>(rows) * Hkv * R <= 0x7fffffffLL, SA_EUNSUPPORTED, "%s: rows*Hkv*T*(Hq/Hkv) too large for one launch", name);
  if (!launch) return SA_OK;

  AttnParams& p = launch->p;
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
  launch->rows = rows;
  return SA_OK;
}

namespace {

sa_status attn_decode_impl(bool dry_run, const void* q, const void* kpool, const void* vpool, int n_pages,
                           const int32_t* page_table, int max_pages, const int32_t* seq_lens, const int32_t* req_idx,
                           int n_req, float* out, int B, int T, int Hq, int Hkv, int D, int page_size, int max_seq_len,
                           int window, float scale, void* workspace, size_t workspace_bytes, void* stream) {
  sa::AttnLaunch l;
  sa_status st = sa::attn_prepare(q, kpool, vpool, n_pages, page_table, max_pages, seq_lens, req_idx, n_req, out, B, T, Hq, Hkv, D,
                                  page_size, max_seq_len, window, scale, workspace, workspace_bytes, dry_run ? nullptr : &l);
  if (st != SA_OK || dry_run || l.rows == 0) return st;
  const AttnParams& p = l.p;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid(p.Hkv, p.nsplit, l.rows);
  if (p.R <= 16)
    sa::launch(SA_K_ATTN_SPLIT, attn_split_kernel<1>, grid, dim3(256), kOccupancyPadBytes, s, p);
  else
    sa::launch(SA_K_ATTN_SPLIT, attn_split_kernel<2>, grid, dim3(256), kOccupancyPadBytes, s, p);
  st = sa::check_launch("attn_decode (split kernel)");
  if (st != SA_OK || p.nsplit == 1) return st;
  sa::launch(SA_K_ATTN_MERGE, attn_merge_kernel, dim3(static_cast<unsigned>(l.rows * p.Hkv * p.R)), dim3(128), 0, s, p);
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

// ---------------------------------------------------------------------------------------------
// attn_decode for callers that cannot allocate: the partial results of the page ranges live in a device array that
// is part of the library's image instead of a caller workspace.
constexpr size_t kScratchBytes = size_t{16} << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// The address of `scratch` on the current device (every device holds its own copy at its own address), looked up
// once per device.  In host code the array's name is only a handle for this lookup, never a device address.
sa_status scratch_address(void** ptr_out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return sa::fail(SA_EHIP, "attn_decode_static: hipGetDevice: %s", hipGetErrorString(e));
  SA_REQUIRE(dev >= 0 && dev < kMaxDevices, SA_EUNSUPPORTED, "attn_decode_static: device index %d beyond %d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return sa::fail(SA_EHIP, "attn_decode_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    }
    g_scratch_ptr[dev] = ptr;
  }
  *ptr_out = g_scratch_ptr[dev];
  return SA_OK;
}

}  // namespace

extern "C" size_t attn_decode_static_max_bytes(void) { return kScratchBytes; }

extern "C" sa_status attn_decode_static(const void* q, const void* kpool, const void* vpool, int n_pages,
                                        const int32_t* page_table, int max_pages, const int32_t* seq_lens,
                                        const int32_t* req_idx, int n_req, float* out, int B, int T, int Hq, int Hkv, int D,
                                        int page_size, int max_seq_len, int window, float scale, void* stream) {
  void* ptr = nullptr;
  sa_status st = scratch_address(&ptr);
  if (st != SA_OK) return st;
  // Everything attn_decode checks, with the array as a workspace of its fixed size: a call whose partial results do not
  // fit is refused (SA_EWORKSPACE) before anything is enqueued.
  st = attn_decode_impl(false, q, kpool, vpool, n_pages, page_table, max_pages, seq_lens, req_idx, n_req, out, B, T, Hq, Hkv, D,
                        page_size, max_seq_len, window, scale, ptr, kScratchBytes, stream);
  if (st == SA_EWORKSPACE)
    return sa::fail(SA_EWORKSPACE,
                    "attn_decode_static: the partial results of this call exceed the library's %zu-byte array; use attn_decode with a "
                    "workspace of attn_decode_workspace_bytes()",
                    kScratchBytes);
  return st;
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
