// Read-rate probe in the attention kernel's launch shape (development aid; stand-alone program).
//
// Every wave streams an equal contiguous share of 8 KiB tiles (4 KiB from a "K" plane and 4 KiB from a "V" plane, as
// decode_stream_kernel does) and does nothing with them, over 28 pairs of planes in turn so that no cache holds the
// data.  It answers one question: would the attention kernel read faster with more bytes in flight per wave?
//   REG d:  d register buffers per wave (d - 1 tiles in flight while one is looked at) -- d = 2 is the kernel's scheme.
//   LDS r:  tiles land in a per-wave LDS ring of r slots through direct-to-LDS loads (global_load_lds_dwordx4), r - 1
//           tiles in flight, no register buffers; then one ds_read_b128 per piece.  policy 0: ordinary, 2: non-temporal.
// usage: read_depth_probe [tiles per launch]   (default 27978 = 229.2 MB, the fused step of BASELINE config 3)
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
#define CK(x)                                                                  \
  do {                                                                         \
    hipError_t e_ = (x);                                                       \
    if (e_ != hipSuccess) {                                                    \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);    \
      exit(1);                                                                 \
    }                                                                          \
  } while (0)

namespace {

struct Share {
  long t0, t1;
};
__device__ inline Share share_of(long tiles, int wpw) {
  const long n_waves = (long)gridDim.x * wpw, w = (long)blockIdx.x * wpw + (threadIdx.x >> 6);
  const long per = (tiles + n_waves - 1) / n_waves;
  const long t0 = w * per;
  return Share{t0, t0 + per < tiles ? t0 + per : tiles};
}

template <int D, int WPW>
__global__ __launch_bounds__(64 * WPW) void reg_kernel(const char* __restrict__ kp, const char* __restrict__ vp, long tiles,
                                                       unsigned* out) {
  const int lane = threadIdx.x & 63;
  const Share s = share_of(tiles, WPW);
  if (s.t0 >= s.t1) return;
  const char* kb = kp + lane * 16;
  const char* vb = vp + lane * 16;
  unsigned acc = 0;
  uint4v bk[D][4], bv[D][4];
#pragma unroll
  for (int d = 0; d < D - 1; ++d) {
    const long t = s.t0 + d < s.t1 ? s.t0 + d : s.t1 - 1;       // never past the share: the planes end with the last one
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bk[d][j] = __builtin_nontemporal_load((const uint4v*)(kb + t * 4096 + j * 1024));
      bv[d][j] = __builtin_nontemporal_load((const uint4v*)(vb + t * 4096 + j * 1024));
    }
  }
  for (long t = s.t0; t < s.t1; t += D) {
#pragma unroll
    for (int u = 0; u < D; ++u) {
      long p = t + u + D - 1;
      p = p < s.t1 ? p : s.t1 - 1;
      const int slot = (u + D - 1) % D;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bk[slot][j] = __builtin_nontemporal_load((const uint4v*)(kb + p * 4096 + j * 1024));
        bv[slot][j] = __builtin_nontemporal_load((const uint4v*)(vb + p * 4096 + j * 1024));
      }
      if (t + u < s.t1) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc += bk[u][j][0] ^ bk[u][j][3] ^ bv[u][j][1] ^ bv[u][j][2];
      }
    }
  }
  if (acc == 0x12345678u) out[0] = acc;                      // keeps the loads alive; the planes never sum to this
}

template <int R, int WPW, int POLICY>
__global__ __launch_bounds__(64 * WPW) void lds_kernel(const char* __restrict__ kp, const char* __restrict__ vp, long tiles,
                                                       unsigned* out) {
  extern __shared__ char lds[];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const Share s = share_of(tiles, WPW);
  if (s.t0 >= s.t1) return;
  const char* kb = kp + lane * 16;
  const char* vb = vp + lane * 16;
  char* ring = lds + wv * (R * 8192);
  const unsigned ring_addr = (unsigned)(uintptr_t)ring + lane * 16;   // LDS byte address of this lane's piece in slot 0
  unsigned acc = 0;
  auto issue = [&](long t, int slot) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kb + t * 4096 + j * 1024),
                                       (__attribute__((address_space(3))) void*)(ring + slot * 8192 + j * 1024), 16, 0, POLICY);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vb + t * 4096 + j * 1024),
                                       (__attribute__((address_space(3))) void*)(ring + slot * 8192 + 4096 + j * 1024), 16, 0, POLICY);
    }
  };
#pragma unroll
  for (int d = 0; d < R - 1; ++d) issue(s.t0 + d < s.t1 ? s.t0 + d : s.t1 - 1, d);
  for (long t = s.t0; t < s.t1; t += R) {
#pragma unroll
    for (int u = 0; u < R; ++u) {
      long p = t + u + R - 1;
      p = p < s.t1 ? p : s.t1 - 1;
      issue(p, (u + R - 1) % R);
      if (t + u < s.t1) {
        // loads retire in order: tile t + u has landed when at most the R - 1 younger tiles' loads are outstanding
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((R - 1) * 8) : "memory");
        // All eight reads and the wait for them in ONE statement with early-clobber outputs: the compiler must neither
        // use a result nor hand out its registers before the data has arrived.
        uint4v x[8];
        asm volatile(
            "ds_read_b128 %0, %8 offset:0\n\tds_read_b128 %1, %8 offset:1024\n\tds_read_b128 %2, %8 offset:2048\n\t"
            "ds_read_b128 %3, %8 offset:3072\n\tds_read_b128 %4, %8 offset:4096\n\tds_read_b128 %5, %8 offset:5120\n\t"
            "ds_read_b128 %6, %8 offset:6144\n\tds_read_b128 %7, %8 offset:7168\n\ts_waitcnt lgkmcnt(0)"
            : "=&v"(x[0]), "=&v"(x[1]), "=&v"(x[2]), "=&v"(x[3]), "=&v"(x[4]), "=&v"(x[5]), "=&v"(x[6]), "=&v"(x[7])
            : "v"(ring_addr + u * 8192)
            : "memory");
#pragma unroll
        for (int j = 0; j < 8; ++j) acc += x[j][0] ^ x[j][3] ^ x[j][1] ^ x[j][2];
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");            // nothing lands in LDS after the wave has gone
  if (acc == 0x12345678u) out[0] = acc;
}

constexpr int PLANES = 28;
char *kbase, *vbase;
unsigned* sink;
size_t plane;
long tiles;

template <class F>
float time_us(F launch) {
  hipEvent_t a, b;
  CK(hipEventCreate(&a));
  CK(hipEventCreate(&b));
  for (int i = 0; i < PLANES; ++i) launch(i);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(a));
  for (int it = 0; it < 5; ++it)
    for (int i = 0; i < PLANES; ++i) launch(i);
  CK(hipEventRecord(b));
  CK(hipEventSynchronize(b));
  CK(hipGetLastError());
  float ms;
  CK(hipEventElapsedTime(&ms, a, b));
  CK(hipEventDestroy(a));
  CK(hipEventDestroy(b));
  return ms * 1e3f / (5 * PLANES);
}

template <int D, int WPW>
void run_reg(int grid) {
  const float us = time_us([&](int i) {
    hipLaunchKernelGGL((reg_kernel<D, WPW>), dim3(grid), dim3(64 * WPW), 0, 0, kbase + (size_t)i * plane, vbase + (size_t)i * plane, tiles, sink);
  });
  printf("REG %d (%d tiles in flight per wave), %d waves per work-group, %4d work-groups:              %6.2f us  %5.0f GB/s\n", D, D - 1, WPW, grid,
         us, 2.0 * plane / us / 1e3);
  fflush(stdout);
}
template <int R, int WPW, int POLICY>
void run_lds(int grid) {
  const int bytes = WPW * R * 8192;                          // at most 160 KiB: checked below against the device limit
  int lim = 0;
  CK(hipDeviceGetAttribute(&lim, hipDeviceAttributeMaxSharedMemoryPerBlock, 0));
  if (bytes > 160 * 1024) {
    printf("LDS %d x %d waves: %d KiB exceeds the LDS of a CU, skipped\n", R, WPW, bytes / 1024);
    return;
  }
  CK(hipFuncSetAttribute((const void*)lds_kernel<R, WPW, POLICY>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  const float us = time_us([&](int i) {
    hipLaunchKernelGGL((lds_kernel<R, WPW, POLICY>), dim3(grid), dim3(64 * WPW), bytes, 0, kbase + (size_t)i * plane, vbase + (size_t)i * plane, tiles,
                       sink);
  });
  printf("LDS %d policy %d (%d tiles in flight per wave), %d waves per work-group, %4d work-groups, %3d KiB LDS: %6.2f us  %5.0f GB/s\n", R, POLICY,
         R - 1, WPW, grid, bytes / 1024, us, 2.0 * plane / us / 1e3);
  fflush(stdout);
}

}  // namespace

int main(int argc, char** argv) {
  tiles = argc > 1 ? atol(argv[1]) : 27978;
  if (tiles < 1024 || tiles > 200000) {
    printf("tiles per launch must be in 1024..200000\n");
    return 2;
  }
  plane = (size_t)tiles * 4096;
  printf("%ld tiles of 8 KiB per launch = %.1f MB, %d plane pairs in turn\n", tiles, 2.0 * plane / 1e6, PLANES);
  CK(hipMalloc(&kbase, plane * PLANES));
  CK(hipMalloc(&vbase, plane * PLANES));
  CK(hipMalloc(&sink, 4));
  CK(hipMemset(kbase, 1, plane * PLANES));
  CK(hipMemset(vbase, 2, plane * PLANES));
  CK(hipMemset(sink, 0, 4));
  run_reg<2, 4>(256);
  run_reg<3, 4>(256);
  run_reg<4, 4>(256);
  run_reg<6, 4>(256);
  run_reg<2, 4>(512);
  run_reg<3, 4>(512);
  run_reg<2, 8>(256);
  run_reg<3, 8>(256);
  run_lds<2, 4, 0>(256);
  run_lds<3, 4, 0>(256);
  run_lds<2, 4, 2>(256);
  run_lds<3, 4, 2>(256);
  run_lds<4, 4, 2>(256);
  run_lds<5, 4, 2>(256);
  run_lds<2, 4, 2>(512);
  run_lds<2, 8, 2>(256);
  run_lds<3, 4, 2>(512);
  run_lds<4, 2, 2>(512);
  run_reg<2, 4>(256);
  CK(hipFree(kbase));
  CK(hipFree(vbase));
  CK(hipFree(sink));
  return 0;
}
