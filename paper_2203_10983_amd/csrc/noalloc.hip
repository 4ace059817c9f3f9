// bns_sample_boundary_noalloc: the selection step of Algorithm 1 for callers that can neither
// allocate device memory nor carry a workspace.  Same kernels as bns_sample_boundary; their scratch
// (keep bits as ballot words, per-tile counts) lives in a fixed array in device memory that the
// library's code object brings along, one copy per GPU.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <mutex>

#include "../../include/bns_gcn.h"
#include "kernels.hpp"

using namespace bns;

namespace {

constexpr int64_t kMaxHalo = BNS_NOALLOC_MAX_HALO;
constexpr size_t kBallotBytes = ((size_t)(kMaxHalo + 63) / 64 + 1) * sizeof(uint64_t);
constexpr size_t kBallotBytesAligned = (kBallotBytes + 255) / 256 * 256;
constexpr size_t kTileBytes = ((size_t)(kMaxHalo + kScanTile - 1) / kScanTile + 4) * sizeof(int32_t);
constexpr size_t kScratchBytes = kBallotBytesAligned + (kTileBytes + 255) / 256 * 256;

// Every GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress: it is never
// passed to a kernel or a copy.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mutex;
unsigned char *g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device (nullptr: not resolved yet)

thread_local char t_error[160] = "";

bns_status fail(bns_status st, const char *msg, const char *detail = "") {
  std::snprintf(t_error, sizeof t_error, "%s%s", msg, detail);
  return st;
}

// Device address of this device's copy of `scratch` (resolved once per device, with it current).
hipError_t scratch_address(unsigned char **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

// Error text of the context-free calls on this thread (read through bns_last_error(NULL)).
const char *bns_noalloc_last_error() { return t_error; }

extern "C" bns_status bns_sample_boundary_noalloc(const int64_t *halo_gid, int32_t n_halo, int32_t part_id,
                                                  uint64_t seed, uint32_t epoch, double p, int32_t *kept_ids,
                                                  int32_t *remap, int32_t *n_kept, void *stream) {
  t_error[0] = '\0';
  if (!(p >= 0.0 && p <= 1.0)) return fail(BNS_EINVAL, "p must lie in [0, 1]");
  if (n_halo < 0) return fail(BNS_EINVAL, "n_halo must not be negative");
  if ((int64_t)n_halo > kMaxHalo)
    return fail(BNS_EOVERFLOW, "n_halo exceeds BNS_NOALLOC_MAX_HALO, the size the fixed scratch array is built for");
  if (!n_kept || (n_halo > 0 && (!halo_gid || !kept_ids || !remap))) return fail(BNS_EINVAL, "null pointer");
  unsigned char *base = nullptr;
  hipError_t e = scratch_address(&base);
  if (e != hipSuccess) {
    (void)hipGetLastError();  // do not leave the code behind for the next launcher's hipGetLastError()
    return fail(BNS_EHIP, "hipGetSymbolAddress(scratch): ", hipGetErrorString(e));
  }
  // Nothing in the scratch has to start at zero: the first kernel writes every ballot word and
  // every tile count that the later ones read, so what an earlier (larger) call left is never seen.
  uint64_t *ballots = reinterpret_cast<uint64_t *>(base);
  int32_t *tile_sums = reinterpret_cast<int32_t *>(base + kBallotBytesAligned);
  const uint64_t threshold = (uint64_t)std::floor(p * 4294967296.0);
  e = sample_boundary(halo_gid, n_halo, seed, epoch, nullptr, (uint32_t)part_id, threshold, ballots, tile_sums,
                      kept_ids, remap, n_kept, nullptr, 0, nullptr, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(BNS_EHIP, "sample_boundary: ", hipGetErrorString(e));
  }
  return BNS_OK;
}
