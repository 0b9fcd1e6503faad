// Stand-alone HBM probe for MI355X: what read bandwidth does the attention kernels' access
// pattern reach by itself, and what does a small write stream cost?  Used to set the achievable
// ceiling that the kernels' numbers are compared with (the nominal peak is 8 TB/s).
//
// The read pattern is exactly the wavefront kernel's: a "page" is 8 tiles of 4 KiB (one per kv
// head) in a K pool and in a V pool; one wavefront handles (branch, head) = npg pages, two pages
// per step, 16 loads of 1 KiB per step (512 B from each page), the next step's loads in flight
// while the current ones are consumed.  Pages are placed sequentially or by a seeded shuffle.
// Optionally every wavefront ends by writing 4 KiB (the size of 8 fp32 output rows).
//
// Build: hipcc --offload-arch=gfx950 -O3 hbm_probe.hip -o hbm_probe      Run: ./hbm_probe
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <random>
#include <vector>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                          \
  do {                                                                    \
    hipError_t e_ = (x);                                                  \
    if (e_ != hipSuccess) {                                               \
      std::printf("%s failed: %s\n", #x, hipGetErrorString(e_));          \
      return 1;                                                           \
    }                                                                     \
  } while (0)

__global__ __launch_bounds__(256) void read_tiles(const char *__restrict__ kp, const char *__restrict__ vp,
                                                  const int *__restrict__ perm, int nitems, int npg,
                                                  uint32_t *out, char *wr, int write_mode) {
  const int item = __builtin_amdgcn_readfirstlane((blockIdx.x * 256 + threadIdx.x) >> 6);
  const int lane = threadIdx.x & 63, m16 = lane & 15, jj = lane >> 4;
  if (item >= nitems) return;
  const int leaf = item >> 3, g = item & 7;
  const int *pl = perm + static_cast<size_t>(leaf) * npg;
  u32x4 acc = {0, 0, 0, 0};
  u32x4 r[2][16];
  auto issue = [&](u32x4 *rr, int b) {
    const size_t ta = (static_cast<size_t>(pl[2 * b]) * 8 + g) * 4096;
    const size_t tb = (static_cast<size_t>(pl[2 * b + 1]) * 8 + g) * 4096;
    const char *k = kp + (m16 < 8 ? ta : tb) + jj * 128 + (m16 & 7) * 16;
    const char *v = vp + (jj < 2 ? ta : tb) + (jj & 1) * 256 + m16 * 16;
#pragma unroll
    for (int s = 0; s < 8; ++s) rr[s] = *reinterpret_cast<const u32x4 *>(k + s * 512);
#pragma unroll
    for (int s = 0; s < 8; ++s) rr[8 + s] = *reinterpret_cast<const u32x4 *>(v + s * 512);
  };
  auto use = [&](u32x4 *rr) {
#pragma unroll
    for (int s = 0; s < 16; ++s) acc ^= rr[s];
  };
  const int nblk = npg / 2;
  issue(r[0], 0);
  int b = 0;
  for (; b + 2 < nblk; b += 2) {
    issue(r[1], b + 1);
    use(r[0]);
    issue(r[0], b + 2);
    use(r[1]);
  }
  if (b + 1 < nblk) {
    issue(r[1], b + 1);
    use(r[0]);
    use(r[1]);
  } else {
    use(r[0]);
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) out[0] = 1;
  if (write_mode) {  // 4 KiB per wavefront, 1 KiB contiguous per instruction
    u32x4 *w = reinterpret_cast<u32x4 *>(wr + static_cast<size_t>(item) * 4096) + lane;
    for (int s = 0; s < 4; ++s) w[s * 64] = acc;
  }
}

__global__ __launch_bounds__(256) void read_stream(const u32x4 *__restrict__ p, size_t n16, uint32_t *out) {
  const size_t tid = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t i = tid; i + 3 * stride < n16; i += 4 * stride) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = p[i + u * stride];
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= v[u];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) out[0] = 1;
}

int main() {
  const int npages = 131072;  // 32 KiB per page and pool -> 4 GiB per pool
  const size_t bytes = static_cast<size_t>(npages) * 32768;
  char *k, *v, *wr;
  uint32_t *o;
  int *dperm;
  CHECK(hipMalloc(&k, bytes));
  CHECK(hipMalloc(&v, bytes));
  CHECK(hipMalloc(&o, 4));
  CHECK(hipMalloc(&wr, static_cast<size_t>(npages) * 4096));
  CHECK(hipMalloc(&dperm, npages * sizeof(int)));
  CHECK(hipMemset(k, 1, bytes));
  CHECK(hipMemset(v, 1, bytes));
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));

  for (int blocks : {512, 2048, 8192}) {
    float best = 1e9f;
    for (int it = 0; it < 4; ++it) {
      CHECK(hipEventRecord(e0));
      read_stream<<<blocks, 256>>>(reinterpret_cast<const u32x4 *>(k), bytes / 16, o);
      CHECK(hipEventRecord(e1));
      CHECK(hipEventSynchronize(e1));
      float ms;
      CHECK(hipEventElapsedTime(&ms, e0, e1));
      best = ms < best ? ms : best;
    }
    std::printf("stream read, %5d workgroups:            %7.1f GB/s\n", blocks, bytes / best / 1e6);
  }
  std::vector<int> perm(npages);
  for (int rnd = 0; rnd < 2; ++rnd) {
    for (int i = 0; i < npages; ++i) perm[i] = i;
    if (rnd) {
      std::mt19937 gen(1);
      std::shuffle(perm.begin(), perm.end(), gen);
    }
    CHECK(hipMemcpy(dperm, perm.data(), npages * sizeof(int), hipMemcpyHostToDevice));
    for (int npg : {8, 16, 64})
      for (int wmode = 0; wmode < 2; ++wmode) {
        const int nitems = npages / npg * 8;
        float best = 1e9f;
        for (int it = 0; it < 3; ++it) {
          CHECK(hipEventRecord(e0));
          read_tiles<<<(nitems + 3) / 4, 256>>>(k, v, dperm, nitems, npg, o, wr, wmode);
          CHECK(hipEventRecord(e1));
          CHECK(hipEventSynchronize(e1));
          float ms;
          CHECK(hipEventElapsedTime(&ms, e0, e1));
          best = ms < best ? ms : best;
        }
        std::printf("tile pattern, %s pages, %3d pages/wave, %s: %7.1f GB/s read\n",
                    rnd ? "shuffled  " : "sequential", npg, wmode ? "4 KiB written per wave" : "no writes            ",
                    2.0 * bytes / best / 1e6);
      }
  }
  return 0;
}
