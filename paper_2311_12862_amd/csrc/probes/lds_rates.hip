// LDS access-rate probe for gfx950 (a developer tool, not part of the library): the four waves of
// one workgroup issue eight independent DS instructions per iteration, each lane at a byte address
// given by the host, and the shader clock gives the cost per wave instruction.  It answers the
// questions the LDS layouts of the tiled kernels depend on: how many bytes per clock reads and
// writes of each width move, and which row pitches keep the fragment reads of the 16x16x32 MFMA
// operands (row = lane % 16, 16 bytes at (lane / 16) * 16; or the transposing 8-byte reads) off
// bank conflicts.  All addresses are checked on the host against the size of the LDS array.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <string>
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr int kLds = 60 * 1024;
constexpr int kIters = 512, kUnroll = 8;
// kind: 0 = read b32, 1 = read b64, 2 = read b128, 3 = read tr16_b64, 4 = write b128, 5 = write b64
#define RD8(INSTR, T)                                                                                     \
  {                                                                                                      \
    T v0, v1, v2, v3, v4, v5, v6, v7;                                                                    \
    asm volatile(INSTR " %0, %8\n" INSTR " %1, %8 offset:4096\n" INSTR " %2, %8 offset:8192\n" INSTR       \
                       " %3, %8 offset:12288\n" INSTR " %4, %8 offset:16384\n" INSTR " %5, %8 offset:20480\n" \
                 INSTR " %6, %8 offset:24576\n" INSTR " %7, %8 offset:28672\ns_waitcnt lgkmcnt(0)"          \
                 : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7) \
                 : "v"(a)                                                                                \
                 : "memory");                                                                            \
    acc += FIRST(v0) + FIRST(v1) + FIRST(v2) + FIRST(v3) + FIRST(v4) + FIRST(v5) + FIRST(v6) + FIRST(v7); \
  }
__device__ __forceinline__ unsigned FIRST(unsigned v) { return v; }
__device__ __forceinline__ unsigned FIRST(u32x2 v) { return v[0]; }
__device__ __forceinline__ unsigned FIRST(u32x4 v) { return v[0]; }
template <int KIND>
__global__ void __launch_bounds__(256) k_probe(const int* __restrict__ addr, long long* __restrict__ out, int slot) {
  __shared__ __align__(16) unsigned char lds[kLds];
  const int lane = threadIdx.x & 63;
  for (int i = threadIdx.x; i < kLds / 4; i += 256) reinterpret_cast<unsigned*>(lds)[i] = i;
  __syncthreads();
  // LDS byte address of this lane (the array starts at LDS offset 0: it is the only shared object)
  const unsigned a = (unsigned)addr[lane];
  unsigned acc = 0;
  long long t0 = clock64();
  for (int it = 0; it < kIters; ++it) {
    if (KIND == 0) RD8("ds_read_b32", unsigned)
    if (KIND == 1) RD8("ds_read_b64", u32x2)
    if (KIND == 2) RD8("ds_read_b128", u32x4)
    if (KIND == 3) RD8("ds_read_b64_tr_b16", u32x2)
    if (KIND == 4) {
      u32x4 w = {acc, (unsigned)it, (unsigned)lane, 1u};
      asm volatile("ds_write_b128 %0, %1\nds_write_b128 %0, %1 offset:4096\nds_write_b128 %0, %1 offset:8192\n"
                   "ds_write_b128 %0, %1 offset:12288\nds_write_b128 %0, %1 offset:16384\n"
                   "ds_write_b128 %0, %1 offset:20480\nds_write_b128 %0, %1 offset:24576\n"
                   "ds_write_b128 %0, %1 offset:28672\ns_waitcnt lgkmcnt(0)" ::"v"(a), "v"(w) : "memory");
      acc += (unsigned)it;
    }
    if (KIND == 5) {
      u32x2 w = {acc, (unsigned)it};
      asm volatile("ds_write_b64 %0, %1\nds_write_b64 %0, %1 offset:4096\nds_write_b64 %0, %1 offset:8192\n"
                   "ds_write_b64 %0, %1 offset:12288\nds_write_b64 %0, %1 offset:16384\n"
                   "ds_write_b64 %0, %1 offset:20480\nds_write_b64 %0, %1 offset:24576\n"
                   "ds_write_b64 %0, %1 offset:28672\ns_waitcnt lgkmcnt(0)" ::"v"(a), "v"(w) : "memory");
      acc += (unsigned)it;
    }
    if (KIND == 6) {
      unsigned w = acc;
      asm volatile("ds_write_b32 %0, %1\nds_write_b32 %0, %1 offset:4096\nds_write_b32 %0, %1 offset:8192\n"
                   "ds_write_b32 %0, %1 offset:12288\nds_write_b32 %0, %1 offset:16384\n"
                   "ds_write_b32 %0, %1 offset:20480\nds_write_b32 %0, %1 offset:24576\n"
                   "ds_write_b32 %0, %1 offset:28672\ns_waitcnt lgkmcnt(0)" ::"v"(a), "v"(w) : "memory");
      acc += (unsigned)it;
    }
  }
  long long t1 = clock64();
  if (acc == 0x12345678u) out[63] = acc;  // keep the work alive
  if (threadIdx.x == 0) out[slot] = t1 - t0;
}
struct Pat { std::string name; int kind; std::vector<int> a; };
int main() {
  std::vector<Pat> pats;
  auto add = [&](std::string n, int kind, auto f) { Pat p{n, kind, std::vector<int>(64)}; for (int l = 0; l < 64; ++l) p.a[l] = f(l); pats.push_back(p); };
  const int sz[7] = {4, 8, 16, 8, 16, 8, 4};
  for (int kind : {0, 1, 2, 3, 4, 5, 6}) {
    add("contiguous", kind, [&](int l) { return l * sz[kind]; });
    add("broadcast", kind, [&](int l) { return 0; });
    for (int stride : {32, 64, 128, 256, 512, 1024})
      if (stride > sz[kind]) add("stride " + std::to_string(stride) + "B", kind, [&](int l) { return l * stride % 4096 + (l * stride / 4096) * sz[kind]; });
  }
  // kernel-2 patterns: A fragment read (b128): row = l%16, 16-byte group l/16, pitch 144 B and others
  for (int pitch : {128, 144, 160, 136, 272, 288})
    add("A-frag pitch " + std::to_string(pitch), 2, [&](int l) { return (l % 16) * pitch + (l / 16) * 16; });
  // B fragment, transposing read: row = 8*(l/16) + (l%16)/4, 8 bytes at (l%4)*8, pitches in bytes
  for (int pitch : {288, 272, 264, 280, 296, 304, 160, 144, 96})
    add("B-tr pitch " + std::to_string(pitch), 3, [&](int l) { return (8 * (l / 16) + (l % 16) / 4) * pitch + (l % 4) * 8; });
  // same with the +4-row half taken first by odd 16-lane groups
  for (int pitch : {288, 160, 96})
    add("B-tr alt pitch " + std::to_string(pitch), 3, [&](int l) { int g = l / 16; return (8 * g + (g & 1) * 4 + (l % 16) / 4) * pitch + (l % 4) * 8; });
  // A store (b128): thread t: seg = t%8, row = t/8, pitch 144; B store: seg = t%16, row = t/16, pitch 288
  for (int pitch : {128, 144, 160})
    add("A-store pitch " + std::to_string(pitch), 4, [&](int l) { return (l / 8) * pitch + (l % 8) * 16; });
  for (int pitch : {144, 160})
    add("A-store(b64) pitch " + std::to_string(pitch), 5, [&](int l) { return (l / 16) * pitch + (l % 16) * 8; });
  for (int pitch : {256, 288})
    add("B-store pitch " + std::to_string(pitch), 4, [&](int l) { return (l / 16) * pitch + (l % 16) * 16; });
  for (auto& p : pats)
    for (int l = 0; l < 64; ++l)
      if (p.a[l] < 0 || p.a[l] + 7 * 4096 + 16 > kLds) { printf("pattern %s lane %d out of range\n", p.name.c_str(), l); return 1; }
  int* d_addr; long long* d_out;
  if (hipMalloc(&d_addr, 64 * sizeof(int)) != hipSuccess || hipMalloc(&d_out, 64 * sizeof(long long)) != hipSuccess) return 2;
  const char* kn[7] = {"read_b32", "read_b64", "read_b128", "read_tr16_b64", "write_b128", "write_b64", "write_b32"};
  for (auto& p : pats) {
    hipMemcpy(d_addr, p.a.data(), 64 * sizeof(int), hipMemcpyHostToDevice);
    for (int rep = 0; rep < 2; ++rep) {
      switch (p.kind) {
        case 0: hipLaunchKernelGGL(k_probe<0>, dim3(1), dim3(256), 0, 0, d_addr, d_out, 0); break;
        case 1: hipLaunchKernelGGL(k_probe<1>, dim3(1), dim3(256), 0, 0, d_addr, d_out, 0); break;
        case 2: hipLaunchKernelGGL(k_probe<2>, dim3(1), dim3(256), 0, 0, d_addr, d_out, 0); break;
        case 3: hipLaunchKernelGGL(k_probe<3>, dim3(1), dim3(256), 0, 0, d_addr, d_out, 0); break;
        case 4: hipLaunchKernelGGL(k_probe<4>, dim3(1), dim3(256), 0, 0, d_addr, d_out, 0); break;
        case 5: hipLaunchKernelGGL(k_probe<5>, dim3(1), dim3(256), 0, 0, d_addr, d_out, 0); break;
        case 6: hipLaunchKernelGGL(k_probe<6>, dim3(1), dim3(256), 0, 0, d_addr, d_out, 0); break;
      }
      if (hipDeviceSynchronize() != hipSuccess) { printf("launch failed\n"); return 3; }
    }
    long long cyc = 0;
    hipMemcpy(&cyc, d_out, sizeof(cyc), hipMemcpyDeviceToHost);
    printf("%-14s %-22s %7.2f clk per wave-instruction (4 waves share the LDS)\n", kn[p.kind], p.name.c_str(),
           (double)cyc / (kIters * kUnroll));
    fflush(stdout);
  }
  return 0;
}
