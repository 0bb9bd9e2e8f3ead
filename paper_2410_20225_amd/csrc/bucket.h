// Counting sort by a small integer key, for inputs in which a few keys are very frequent (the
// lowest dependency levels hold most cells; token ids follow a Zipf law).  Every workgroup
// counts its slice of the items in an LDS histogram first and touches each global counter
// once, so a hot key costs one global atomic per workgroup instead of one per wave.
#pragma once
#include "engine.h"

namespace tdf {
namespace {   // every translation unit that includes this header gets its own copy of the kernels

constexpr uint32_t BUCKET_MAX_KEYS = 40000;   // LDS histogram entries (156 KB of the 160)
constexpr int BUCKET_BLOCKS = 256;
constexpr int BUCKET_THREADS = 512;

// count[k] += number of items with key k (keys >= n_keys are skipped)
__device__ inline void bucket_hist_lds(uint32_t* hist, const uint32_t* keys, uint32_t lo, uint32_t hi, uint32_t n_keys) {
  for (uint32_t k = threadIdx.x; k < n_keys; k += blockDim.x) hist[k] = 0;
  __syncthreads();
  for (uint32_t base = lo; base < hi; base += blockDim.x) {   // uniform trip count for the workgroup
    const uint32_t i = base + threadIdx.x;
    const uint32_t k = i < hi ? keys[i] : 0xFFFFFFFFu;
    (void)wave_alloc_keyed(k < n_keys, k < n_keys ? k : 0, hist);
  }
  __syncthreads();
}

__global__ void __launch_bounds__(BUCKET_THREADS) k_bucket_count(const uint32_t* keys, uint32_t n, uint32_t n_keys,
                                                                 uint32_t* count) {
  extern __shared__ uint32_t hist[];
  const uint32_t per = (n + gridDim.x - 1) / gridDim.x;
  const uint32_t lo = min(n, blockIdx.x * per), hi = min(n, lo + per);
  bucket_hist_lds(hist, keys, lo, hi, n_keys);
  for (uint32_t k = threadIdx.x; k < n_keys; k += blockDim.x)
    if (hist[k]) atomicAdd(&count[k], hist[k]);
}

// Item i goes to position off[key] + (its rank among the items of that key); sink(i, position).
// fill[] must be zero on entry.  The order of equal keys is not fixed.
template <class Sink>
__global__ void __launch_bounds__(BUCKET_THREADS) k_bucket_place(const uint32_t* keys, uint32_t n, uint32_t n_keys,
                                                                 const uint32_t* off, uint32_t* fill, Sink sink) {
  extern __shared__ uint32_t hist[];
  const uint32_t per = (n + gridDim.x - 1) / gridDim.x;
  const uint32_t lo = min(n, blockIdx.x * per), hi = min(n, lo + per);
  bucket_hist_lds(hist, keys, lo, hi, n_keys);
  // the workgroup's range of every key it holds; the LDS entry becomes the next free position
  for (uint32_t k = threadIdx.x; k < n_keys; k += blockDim.x)
    if (hist[k]) hist[k] = off[k] + atomicAdd(&fill[k], hist[k]);
  __syncthreads();
  for (uint32_t base = lo; base < hi; base += blockDim.x) {
    const uint32_t i = base + threadIdx.x;
    const uint32_t k = i < hi ? keys[i] : 0xFFFFFFFFu;
    const bool on = k < n_keys;
    const uint32_t pos = wave_alloc_keyed(on, on ? k : 0, hist);
    if (on) sink(i, pos);
  }
}

inline bool bucket_fits(uint32_t n_keys) { return n_keys <= BUCKET_MAX_KEYS; }

// LDS above 48 KB needs an opt-in per kernel; `fn` is the kernel's address.
inline void bucket_lds_opt_in(const void* fn, uint32_t n_keys) {
  if (n_keys * 4u > 48u * 1024u)
    (void)hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(BUCKET_MAX_KEYS * 4));
}

}  // namespace
}  // namespace tdf
