// si_rehash_check for callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops): the partial sums live in a file-scope device array instead of a
// caller-provided scratch buffer.  Included by si_api.hip inside its extern "C" block.
#pragma once

// The partial sums live in this array.
// In host code the array's name is only a handle for hipGetSymbolAddress; its device address is
// resolved once per device and used from then on.
static __device__ __align__(256) unsigned char scratch[SI_REHASH_STATIC_SCRATCH_BYTES];
static_assert(SI_REHASH_STATIC_SCRATCH_BYTES >= si::kCosMaxBlocks * 3 * sizeof(double), "room for every block's partial sums");

static si_status static_scratch_ptr(void** out) {
  static std::mutex mu;
  static void* per_device[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return SI_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!per_device[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SI_ERR_HIP;
    per_device[dev] = ptr;
  }
  *out = per_device[dev];
  return SI_OK;
}

si_status si_init_device(void) {
  void* ptr = nullptr;
  return static_scratch_ptr(&ptr);
}

si_status si_rehash_check_static(const void* feat_t, const void* feat_prev, int64_t n, int32_t dtype, float thresh,
                                 double* cos_dev, int32_t* decision_dev, void* stream) {
  if (n < 0 || n > SI_REHASH_STATIC_MAX_N) return SI_ERR_SHAPE;
  void* ptr = nullptr;
  si_status s = static_scratch_ptr(&ptr);
  if (s != SI_OK) return s;
  // every block overwrites its own partial sums and the finishing kernel reads exactly those: nothing
  // has to be cleared between calls
  return si_rehash_check(feat_t, feat_prev, n, dtype, thresh, cos_dev, decision_dev, ptr, stream);
}

