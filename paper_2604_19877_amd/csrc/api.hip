// Error reporting, launch profiling and the calibration kernels (plain copy, tile streams) of libsamixers.
#include <mutex>
#include <vector>

#include "common.h"
#include "delta_device.h"

namespace {

thread_local char g_error[512] = "";

struct EventPair {
  hipEvent_t start, stop;
};
std::mutex g_prof_mutex;
bool g_prof_on = false;
std::vector<EventPair> g_prof[SA_K_COUNT];

}  // namespace

namespace sa {

sa_status fail(sa_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}

sa_status check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SA_EHIP, "%s: %s", what, hipGetErrorString(e));
  return SA_OK;
}

bool prof_enabled() { return g_prof_on; }

void prof_record(int kernel_id, hipEvent_t start, hipEvent_t stop) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  g_prof[kernel_id].push_back({start, stop});
}

}  // namespace sa

extern "C" {

const char* sa_last_error(void) { return g_error; }

int sa_version(void) { return 100; }

void sa_prof_enable(int on) { g_prof_on = on != 0; }

sa_status sa_prof_read(int kernel, int* n_launches, float* total_ms, float* ms_each, int capacity) {
  SA_REQUIRE(kernel >= 0 && kernel < SA_K_COUNT, SA_EINVAL, "sa_prof_read: unknown kernel id %d", kernel);
  SA_REQUIRE(n_launches && total_ms, SA_EINVAL, "sa_prof_read: null output pointer");
  std::vector<EventPair> taken;
  {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    taken.swap(g_prof[kernel]);
  }
  float sum = 0.f;
  sa_status st = SA_OK;
  int at = 0;
  for (const EventPair& p : taken) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(p.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, p.start, p.stop);
    if (e != hipSuccess) st = sa::fail(SA_EHIP, "sa_prof_read: %s", hipGetErrorString(e));
    sum += ms;
    if (ms_each && at < capacity) ms_each[at] = ms;
    ++at;
    (void)hipEventDestroy(p.start);
    (void)hipEventDestroy(p.stop);
  }
  *n_launches = static_cast<int>(taken.size());
  *total_ms = sum;
  return st;
}

}  // extern "C"

namespace {

// Grid-stride copy, 16 bytes per lane per iteration (the tail of sa_copy_bytes, and the state conversions).
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Copy in 64 KiB tiles, one per workgroup, the way the recurrent step moves a state tile: all 16 non-temporal 16-byte
// loads of a lane are requested before the first store, rows are walked from a start that differs between neighbouring
// workgroups, and the tile list is visited in four interleaved quarters.  This is the copy the bandwidth figures are
// compared with (a plain grid-stride copy reaches 4.6 TB/s on MI355X, less than any kernel of the library).
__global__ __launch_bounds__(256) void copy_tiles_kernel(const float* __restrict__ src, float* __restrict__ dst) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int c8 = lane & 7, r8 = lane >> 3;
  const size_t tile = static_cast<size_t>(interleaved_tile(blockIdx.x, gridDim.x));
  const int turn4 = 4 * (blockIdx.x & 3);
  const size_t at = tile * (128 * 128) + (r8 * 16) * 128 + wave * 32 + c8 * 4;
  float4 s[16];
#pragma unroll
  for (int m = 0; m < 16; ++m) s[m] = load_state(src + at + ((m + turn4) & 15) * 128);
#pragma unroll
  for (int m = 0; m < 16; ++m) store_state(dst + at + ((m + turn4) & 15) * 128, s[m]);
}

}  // namespace

extern "C" sa_status sa_copy_bytes(const void* src, void* dst, size_t n_bytes, void* stream) {
  SA_REQUIRE(src && dst, SA_EINVAL, "sa_copy_bytes: null pointer");
  SA_REQUIRE(sa::aligned(src, 16) && sa::aligned(dst, 16) && n_bytes % 16 == 0, SA_EINVAL,
             "sa_copy_bytes: pointers and size must be multiples of 16 bytes");
  if (n_bytes == 0) return SA_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  constexpr size_t kTile = 64 * 1024;
  const size_t n_tiles = n_bytes / kTile;
  SA_REQUIRE(n_tiles <= 0x7fffffffULL, SA_EUNSUPPORTED, "sa_copy_bytes: more than 2^31 tiles of 64 KiB");
  if (n_tiles)
    sa::launch(SA_K_COPY, copy_tiles_kernel, dim3(static_cast<unsigned>(n_tiles)), dim3(256), 0, s, static_cast<const float*>(src),
               static_cast<float*>(dst));
  const size_t done = n_tiles * kTile, n16 = (n_bytes - done) / 16;
  if (n16) {
    size_t blocks = (n16 + 255) / 256;
    hipLaunchKernelGGL(copy_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s,
                       reinterpret_cast<const uint4*>(static_cast<const char*>(src) + done),
                       reinterpret_cast<uint4*>(static_cast<char*>(dst) + done), n16);
  }
  return sa::check_launch("sa_copy_bytes");
}

namespace {

// The memory traffic of the recurrent decode step and nothing else: one workgroup per 64 KiB tile, the lane
// pattern and non-temporal accesses of delta_step_kernel (lane (r8, c8) of wavefront w owns columns
// 32w + 4c8 .. +3 of rows 16 r8 .. 16 r8 + 15, walked from a row that differs between neighbouring workgroups, and
// the tile list is visited in four interleaved quarters).  KIND 0 reads the tile, 1 writes it, 2 reads, scales and
// writes it back.
template <int KIND>
__global__ __launch_bounds__(256) void stream_tiles_kernel(float* tiles, float factor) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int c8 = lane & 7, r8 = lane >> 3;
  const int tile = interleaved_tile(blockIdx.x, gridDim.x);
  const int turn4 = 4 * (blockIdx.x & 3);
  float* p = tiles + static_cast<size_t>(tile) * (128 * 128) + (r8 * 16) * 128 + wave * 32 + c8 * 4;
  float4 s[16];
  if (KIND != 1) {
#pragma unroll
    for (int m = 0; m < 16; ++m) s[m] = load_state(p + ((m + turn4) & 15) * 128);
  }
  if (KIND == 0) {
    float acc = 0.f;
#pragma unroll
    for (int m = 0; m < 16; ++m) acc += (s[m].x + s[m].y) + (s[m].z + s[m].w);
    if (acc == factor) p[0] = acc;  // keeps the loads alive; `factor` is chosen so that this never holds
    return;
  }
#pragma unroll
  for (int m = 0; m < 16; ++m) {
    if (KIND == 1) {
      s[m] = float4{factor, factor, factor, factor};
    } else {
      s[m].x *= factor;
      s[m].y *= factor;
      s[m].z *= factor;
      s[m].w *= factor;
    }
    store_state(p + ((m + turn4) & 15) * 128, s[m]);
  }
}

}  // namespace

extern "C" sa_status sa_stream_tiles(int kind, float* tiles, int n_tiles, void* stream) {
  SA_REQUIRE(kind >= 0 && kind <= 2, SA_EINVAL, "sa_stream_tiles: kind=%d not in {0 read, 1 write, 2 read-modify-write}", kind);
  SA_REQUIRE(n_tiles >= 0, SA_EINVAL, "sa_stream_tiles: n_tiles=%d is negative", n_tiles);
  if (n_tiles == 0) return SA_OK;
  SA_REQUIRE(tiles && sa::aligned(tiles, 16), SA_EINVAL, "sa_stream_tiles: null or misaligned pointer");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid(static_cast<unsigned>(n_tiles));
  if (kind == 0)
    sa::launch(SA_K_STREAM, stream_tiles_kernel<0>, grid, dim3(256), 0, s, tiles, 3.0e38f);
  else if (kind == 1)
    sa::launch(SA_K_STREAM, stream_tiles_kernel<1>, grid, dim3(256), 0, s, tiles, 0.01f);
  else
    sa::launch(SA_K_STREAM, stream_tiles_kernel<2>, grid, dim3(256), 0, s, tiles, 0.999f);
  return sa::check_launch("sa_stream_tiles");
}

namespace {

bool state_shape_ok(int dk, int dv) { return (dk == 64 && dv == 64) || (dk == 128 && dv == 128); }

// Both directions are the same copy while a tile is row-major [dk][dv].
sa_status state_convert(const char* name, const float* src, float* dst, int n_tiles, int dk, int dv, void* stream) {
  SA_REQUIRE(state_shape_ok(dk, dv), SA_EUNSUPPORTED, "%s: (dk,dv)=(%d,%d) not in {(64,64),(128,128)}", name, dk, dv);
  SA_REQUIRE(n_tiles >= 0, SA_EINVAL, "%s: n_tiles=%d is negative", name, n_tiles);
  if (n_tiles == 0) return SA_OK;
  SA_REQUIRE(src && dst, SA_EINVAL, "%s: null pointer", name);
  SA_REQUIRE(sa::aligned(src, 16) && sa::aligned(dst, 16), SA_EINVAL, "%s: misaligned pointer", name);
  const size_t n_bytes = static_cast<size_t>(n_tiles) * dk * dv * sizeof(float);
  const char* a = reinterpret_cast<const char*>(src);
  const char* b = reinterpret_cast<const char*>(dst);
  SA_REQUIRE(a + n_bytes <= b || b + n_bytes <= a, SA_EINVAL, "%s: source and destination overlap", name);
  const size_t n16 = n_bytes / 16;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  sa::launch(SA_K_COPY, copy_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, static_cast<hipStream_t>(stream),
             reinterpret_cast<const uint4*>(src), reinterpret_cast<uint4*>(dst), n16);
  return sa::check_launch(name);
}

}  // namespace

extern "C" size_t sa_state_tile_bytes(int dk, int dv) {
  return state_shape_ok(dk, dv) ? static_cast<size_t>(dk) * dv * sizeof(float) : 0;
}

extern "C" sa_status sa_state_pack(const float* rowmajor, float* tiles, int n_tiles, int dk, int dv, void* stream) {
  return state_convert("sa_state_pack", rowmajor, tiles, n_tiles, dk, dv, stream);
}

extern "C" sa_status sa_state_unpack(const float* tiles, float* rowmajor, int n_tiles, int dk, int dv, void* stream) {
  return state_convert("sa_state_unpack", tiles, rowmajor, n_tiles, dk, dv, stream);
}
