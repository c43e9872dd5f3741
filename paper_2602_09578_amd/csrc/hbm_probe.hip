// hbm_probe: plain streaming kernels of known size on the same GPU as the library.
// Two uses: (1) the practical HBM read ceiling for this library's access granularity
// (whole 4 KB blocks, in order or at random, plain or non-temporal 16-byte loads), against
// which the attention kernels' achieved bandwidth is read; (2) a copy kernel of known size
// as the reference reading for the FETCH_SIZE / WRITE_SIZE hardware counters.
// (3) `kv`: a load-only replica of the suffix attention kernel's access pattern (K: 16 rows
// x 64 B per instruction over two pages, V: 2 x 512 B per instruction) against 1 KB-contiguous
// instructions, with cached or non-temporal loads.
// Usage: hbm_probe [read|copy|kv] (default: read sweeps).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <numeric>
#include <algorithm>
#include <random>
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
template <bool NT> __device__ __forceinline__ u32x4 ld(const u32x4* p) {
  if (NT) return __builtin_nontemporal_load(p); else return *p;
}
// each wave reads whole 4 KB blocks (4 x 1 KB instructions), block ids from a table
template <bool NT, int U>
__global__ __launch_bounds__(256) void gather_kernel(const u32x4* __restrict__ p, const int* __restrict__ tbl, int nblk, unsigned* out) {
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * 256 + threadIdx.x) >> 6;
  const int nwaves = gridDim.x * 4;
  u32x4 acc = {0, 0, 0, 0};
  for (int b = wave * U; b < nblk; b += nwaves * U) {
    u32x4 v[U][4];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int id = (b + u < nblk) ? tbl[b + u] : tbl[0];
      const u32x4* q = p + (size_t)id * 256 + lane;
#pragma unroll
      for (int k = 0; k < 4; ++k) v[u][k] = ld<NT>(q + 64 * k);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int k = 0; k < 4; ++k) acc ^= v[u][k];
  }
  unsigned r = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  if (r == 0x12345678u) out[0] = r;
}
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
template <bool NT, int U>
int run(const char* name, const u32x4* a, const int* tbl, int nblk, unsigned* out, int grid, int reps) {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  gather_kernel<NT, U><<<grid, 256>>>(a, tbl, nblk, out);
  CK(hipEventRecord(e0));
  for (int r = 0; r < reps; ++r) gather_kernel<NT, U><<<grid, 256>>>(a, tbl, nblk, out);
  CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  printf("%-28s grid %5d: %.0f GB/s\n", name, grid, (double)nblk * 4096 / (ms / reps * 1e-3) / 1e9);
  return 0;
}
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ p, u32x4* __restrict__ q, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) q[i] = p[i];
}
int copy_main() {
  const size_t bytes = 1024L << 20;   // 1 GiB read + 1 GiB written per launch
  u32x4 *a, *b;
  CK(hipMalloc(&a, bytes)); CK(hipMalloc(&b, bytes));
  CK(hipMemset(a, 1, bytes)); CK(hipMemset(b, 2, bytes));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  copy_kernel<<<2048, 256>>>(a, b, bytes / 16);
  CK(hipEventRecord(e0));
  for (int r = 0; r < 5; ++r) copy_kernel<<<2048, 256>>>(a, b, bytes / 16);
  CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  printf("copy_kernel: %zu bytes read and %zu bytes written per launch, %.0f GB/s read+write\n", bytes, bytes,
         2.0 * bytes / (ms / 5 * 1e-3) / 1e9);
  return 0;
}
// ---- load-only replica of the suffix attention kernel's access pattern -------------------------
template <bool NT> __device__ __forceinline__ u32x4 ldc(const char* p) {
  if (NT) return __builtin_nontemporal_load((const u32x4*)p); else return *(const u32x4*)p;
}
// MODE 0: suffix-kernel pattern. MODE 1: each instruction reads 1 KB contiguous (K: 4 instr per page)
template <bool NTK, bool NTV, int MODE>
__global__ __launch_bounds__(256) void kv_kernel(const char* __restrict__ k, const char* __restrict__ v, const int* __restrict__ tbl, int npairs, int hkv, unsigned* out) {
  const int lane = threadIdx.x & 63, i = lane & 15, j = lane >> 4;
  const int wave = (blockIdx.x * 256 + threadIdx.x) >> 6;
  const int nwaves = gridDim.x * 4;
  const size_t page_bytes = (size_t)hkv * 4096;
  u32x4 acc = {0, 0, 0, 0};
  for (int b = wave; b < npairs * hkv; b += nwaves) {
    const int pr = b / hkv, kvh = b % hkv;
    const int p0 = tbl[2 * pr], p1 = tbl[2 * pr + 1];
    u32x4 kr[8], vr[8];
    if (MODE == 0) {
      const char* kp = k + (size_t)(i < 8 ? p0 : p1) * page_bytes + kvh * 4096 + ((8 * ((i >> 2) & 1) + (i & 3)) * 256 + j * 16);
      const char* vp = v + (size_t)(j < 2 ? p0 : p1) * page_bytes + kvh * 4096 + (i * 32 + (j & 1) * 16);
#pragma unroll
      for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) kr[T * 4 + kk] = ldc<NTK>(kp + T * 1024 + kk * 64);
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) vr[ct] = ldc<NTV>(vp + ct * 512);
    } else {
      const char* k0 = k + (size_t)p0 * page_bytes + kvh * 4096 + lane * 16;
      const char* k1 = k + (size_t)p1 * page_bytes + kvh * 4096 + lane * 16;
      const char* v0 = v + (size_t)p0 * page_bytes + kvh * 4096 + lane * 16;
      const char* v1 = v + (size_t)p1 * page_bytes + kvh * 4096 + lane * 16;
#pragma unroll
      for (int q = 0; q < 4; ++q) { kr[q] = ldc<NTK>(k0 + q * 1024); kr[4 + q] = ldc<NTK>(k1 + q * 1024); }
#pragma unroll
      for (int q = 0; q < 4; ++q) { vr[q] = ldc<NTV>(v0 + q * 1024); vr[4 + q] = ldc<NTV>(v1 + q * 1024); }
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) acc ^= kr[q] ^ vr[q];
  }
  unsigned r = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  if (r == 0x12345678u) out[0] = r;
}
template <bool NTK, bool NTV, int MODE>
int run_kv(const char* name, const char* k, const char* v, const int* tbl, int npairs, int hkv, unsigned* out, int grid) {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  kv_kernel<NTK, NTV, MODE><<<grid, 256>>>(k, v, tbl, npairs, hkv, out);
  CK(hipEventRecord(e0));
  for (int r = 0; r < 5; ++r) kv_kernel<NTK, NTV, MODE><<<grid, 256>>>(k, v, tbl, npairs, hkv, out);
  CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  printf("%-34s grid %5d: %.0f GB/s\n", name, grid, (double)npairs * hkv * 16384 / (ms / 5 * 1e-3) / 1e9);
  return 0;
}
int kv_main() {
  const int hkv = 4, npages = 180000;   // ~2.9 GB K + 2.9 GB V
  const size_t bytes = (size_t)npages * hkv * 4096;
  char *k, *v; unsigned* out; int* tbl;
  CK(hipMalloc(&k, bytes)); CK(hipMalloc(&v, bytes)); CK(hipMalloc(&out, 4)); CK(hipMalloc(&tbl, npages * 4));
  CK(hipMemset(k, 1, bytes)); CK(hipMemset(v, 1, bytes));
  std::vector<int> ids(npages); std::iota(ids.begin(), ids.end(), 0);
  std::mt19937 rng(1); std::shuffle(ids.begin(), ids.end(), rng);
  CK(hipMemcpy(tbl, ids.data(), npages * 4, hipMemcpyHostToDevice));
  const int npairs = npages / 2;
  for (int grid : {512, 1024}) {
    if (run_kv<true, true, 0>("suffix pattern, K nt, V nt", k, v, tbl, npairs, hkv, out, grid)) return 1;
    if (run_kv<false, true, 0>("suffix pattern, K plain, V nt", k, v, tbl, npairs, hkv, out, grid)) return 1;
    if (run_kv<false, false, 0>("suffix pattern, K plain, V plain", k, v, tbl, npairs, hkv, out, grid)) return 1;
    if (run_kv<true, true, 1>("1 KB per instr, K nt, V nt", k, v, tbl, npairs, hkv, out, grid)) return 1;
    if (run_kv<false, false, 1>("1 KB per instr, plain", k, v, tbl, npairs, hkv, out, grid)) return 1;
  }
  return 0;
}

int main(int argc, char** argv) {
  if (argc > 1 && argv[1][0] == 'c') return copy_main();
  if (argc > 1 && argv[1][0] == 'k') return kv_main();
  const size_t bytes = 6144L << 20;
  const int nblk = bytes / 4096;
  u32x4* a; unsigned* out; int *t_seq, *t_rnd;
  CK(hipMalloc(&a, bytes)); CK(hipMalloc(&out, 4)); CK(hipMalloc(&t_seq, nblk * 4)); CK(hipMalloc(&t_rnd, nblk * 4));
  CK(hipMemset(a, 1, bytes));
  std::vector<int> ids(nblk); std::iota(ids.begin(), ids.end(), 0);
  CK(hipMemcpy(t_seq, ids.data(), nblk * 4, hipMemcpyHostToDevice));
  std::mt19937 rng(1); std::shuffle(ids.begin(), ids.end(), rng);
  CK(hipMemcpy(t_rnd, ids.data(), nblk * 4, hipMemcpyHostToDevice));
  for (int grid : {512, 1024, 2048, 4096}) {
    if (run<false, 2>("seq plain U2", a, t_seq, nblk, out, grid, 5)) return 1;
    if (run<true, 2>("seq nt U2", a, t_seq, nblk, out, grid, 5)) return 1;
    if (run<true, 4>("seq nt U4", a, t_seq, nblk, out, grid, 5)) return 1;
    if (run<false, 2>("random-4K plain U2", a, t_rnd, nblk, out, grid, 5)) return 1;
    if (run<true, 2>("random-4K nt U2", a, t_rnd, nblk, out, grid, 5)) return 1;
    if (run<true, 4>("random-4K nt U4", a, t_rnd, nblk, out, grid, 5)) return 1;
  }
  return 0;
}
