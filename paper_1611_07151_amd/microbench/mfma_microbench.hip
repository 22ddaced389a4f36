// Micro-benchmarks of the gfx950 properties the convolution kernels are designed around.
// Not part of libsq.so.  Build and run on the GPU:
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o mfma_microbench paper_1611_07151_amd/microbench/mfma_microbench.hip && ./mfma_microbench
// Part 1: lane layout of the fp32 / bf16 MFMA builtins, MFMA-only throughput, copy bandwidth.
// Part 2: does vector-ALU work overlap with fp32 MFMA?  (V extra v_fma per MFMA)
// Part 3: cost of software-pipelined LDS reads next to fp32 MFMA (L ds_read_b32 per 4 MFMAs).
// Part 4: two wavefronts per SIMD doing different things: one issues MFMAs only, the other
//         vector-ALU work (or LDS writes, or global stores) only.  Do the two streams overlap?
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)

namespace part1 {

__global__ void k32(const float* A, const float* B, float* D) { // A[32][2], B[2][32], D[32][32]
  int l = threadIdx.x; f16v acc = {0};
  float a = A[(l%32)*2 + l/32]; float b = B[(l/32)*32 + l%32];
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0,0,0);
  for (int r=0;r<16;++r){ int i = 8*(r/4) + 4*(l/32) + r%4; int j = l%32; D[i*32+j] = acc[r]; }
}
__global__ void k16(const float* A, const float* B, float* D) { // A[16][4], B[4][16], D[16][16]
  int l = threadIdx.x; f4v acc = {0};
  float a = A[(l%16)*4 + l/16]; float b = B[(l/16)*16 + l%16];
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc, 0,0,0);
  for (int r=0;r<4;++r){ int i = 4*(l/16) + r; int j = l%16; D[i*16+j] = acc[r]; }
}
__global__ void kb32(const float* A, const float* B, float* D) { // A[32][16], B[16][32]
  int l = threadIdx.x; f16v acc = {0}; bf8v a, b;
  for (int t=0;t<8;++t){ int k = 8*(l/32)+t; a[t] = (__bf16)A[(l%32)*16 + k]; b[t] = (__bf16)B[k*32 + l%32]; }
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0,0,0);
  for (int r=0;r<16;++r){ int i = 8*(r/4) + 4*(l/32) + r%4; int j = l%32; D[i*32+j] = acc[r]; }
}
__global__ void kb16(const float* A, const float* B, float* D) { // A[16][32], B[32][16]
  int l = threadIdx.x; f4v acc = {0}; bf8v a, b;
  for (int t=0;t<8;++t){ int k = 8*(l/16)+t; a[t] = (__bf16)A[(l%16)*32 + k]; b[t] = (__bf16)B[k*16 + l%16]; }
  acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0,0,0);
  for (int r=0;r<4;++r){ int i = 4*(l/16) + r; int j = l%16; D[i*16+j] = acc[r]; }
}
// throughput: each wave issues ITER*4 independent-chain MFMAs
template<int KIND> __global__ __launch_bounds__(256) void peak(float* out, int iters) {
  f16v c0={0},c1={0},c2={0},c3={0}; f4v d0={0},d1={0},d2={0},d3={0};
  float a = threadIdx.x*0.001f, b = 1.0f;
  for (int it=0; it<iters; ++it) {
    if (KIND==0) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a,b,c0,0,0,0); c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a,b,c1,0,0,0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a,b,c2,0,0,0); c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(a,b,c3,0,0,0);
    } else {
      d0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a,b,d0,0,0,0); d1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a,b,d1,0,0,0);
      d2 = __builtin_amdgcn_mfma_f32_16x16x4f32(a,b,d2,0,0,0); d3 = __builtin_amdgcn_mfma_f32_16x16x4f32(a,b,d3,0,0,0);
    }
  }
  float s = 0; for (int r=0;r<16;++r) s += c0[r]+c1[r]+c2[r]+c3[r]; for (int r=0;r<4;++r) s += d0[r]+d1[r]+d2[r]+d3[r];
  if (s == 12345.678f) out[0] = s;
}
__global__ __launch_bounds__(256) void copyk(const float4* __restrict__ in, float4* __restrict__ out, size_t n) {
  for (size_t i = (size_t)blockIdx.x*blockDim.x+threadIdx.x; i<n; i += (size_t)gridDim.x*blockDim.x) out[i] = in[i];
}
static void check(const char* name, std::vector<float>&A, std::vector<float>&B, std::vector<float>&D, int M,int N,int K, bool bf){
  double maxe=0; for(int i=0;i<M;++i)for(int j=0;j<N;++j){ double s=0; for(int k=0;k<K;++k){ float a=A[i*K+k], b=B[k*N+j]; s+= (double)a*b;} maxe = fmax(maxe, fabs(s-D[i*N+j])); }
  printf("%s max err %.3g %s\n", name, maxe, maxe < (bf?0.5:1e-4) ? "LAYOUT_OK":"LAYOUT_MISMATCH");
}
int run_part(){
  hipDeviceProp_t p; CK(hipGetDeviceProperties(&p,0));
  printf("device %s CUs %d clock %d kHz memclk %d kHz L2 %d LDS/block %zu arch %s\n", p.name, p.multiProcessorCount, p.clockRate, p.memoryClockRate, p.l2CacheSize, p.sharedMemPerBlock, p.gcnArchName);
  int maxLds=0; hipDeviceGetAttribute(&maxLds, hipDeviceAttributeMaxSharedMemoryPerBlock, 0); printf("max LDS per block %d\n", maxLds);
  float *dA,*dB,*dD; CK(hipMalloc(&dA,4096*4)); CK(hipMalloc(&dB,4096*4)); CK(hipMalloc(&dD,4096*4));
  auto run=[&](const char*name,int M,int N,int K,int kind){ std::vector<float>A(M*K),B(K*N),D(M*N);
    for(auto&v:A) v = (float)((rand()%17)-8)/4.f; for(auto&v:B) v=(float)((rand()%13)-6)/2.f;
    CK(hipMemcpy(dA,A.data(),A.size()*4,hipMemcpyHostToDevice)); CK(hipMemcpy(dB,B.data(),B.size()*4,hipMemcpyHostToDevice));
    if(kind==0) k32<<<1,64>>>(dA,dB,dD); else if(kind==1) k16<<<1,64>>>(dA,dB,dD); else if(kind==2) kb32<<<1,64>>>(dA,dB,dD); else kb16<<<1,64>>>(dA,dB,dD);
    CK(hipDeviceSynchronize()); CK(hipMemcpy(D.data(),dD,D.size()*4,hipMemcpyDeviceToHost)); check(name,A,B,D,M,N,K,kind>=2); };
  run("mfma_f32_32x32x2f32",32,32,2,0); run("mfma_f32_16x16x4f32",16,16,4,1); run("mfma_f32_32x32x16_bf16",32,32,16,2); run("mfma_f32_16x16x32_bf16",16,16,32,3);
  hipEvent_t e0,e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  for (int kind=0; kind<2; ++kind) for (int wpc : {4, 8}) {
    int iters = 20000; int blocks = p.multiProcessorCount * wpc / 4;
    if(kind==0) peak<0><<<blocks,256>>>(dD, 100); else peak<1><<<blocks,256>>>(dD,100);
    CK(hipDeviceSynchronize()); CK(hipEventRecord(e0));
    if(kind==0) peak<0><<<blocks,256>>>(dD, iters); else peak<1><<<blocks,256>>>(dD,iters);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); float ms; CK(hipEventElapsedTime(&ms,e0,e1));
    double flop = (double)blocks*4*iters*4*(kind==0?4096.0:2048.0);
    printf("peak %s waves/CU %d: %.3f ms %.1f TFLOP/s\n", kind==0?"32x32x2":"16x16x4", wpc, ms, flop/ms/1e9);
  }
  size_t n = (size_t)1<<30; float4 *src,*dst; CK(hipMalloc(&src,n)); CK(hipMalloc(&dst,n)); CK(hipMemset(src,1,n));
  for (int rep=0; rep<3; ++rep){ CK(hipEventRecord(e0)); copyk<<<p.multiProcessorCount*8,256>>>(src,dst,n/16); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); float ms; CK(hipEventElapsedTime(&ms,e0,e1)); printf("copy 1GiB: %.3f ms  %.1f GB/s (read+write)\n", ms, 2.0*n/ms/1e6);}  
  printf("probe done\n"); return 0;
}

}  // namespace part1

namespace part2 {
// per MFMA: V independent VALU fma ops (on 4 chains), L ds_read_b32
template<int V, int L, int KIND> __global__ __launch_bounds__(256) void k(float* out, int iters) {
  __shared__ float lds[4096];
  for (int i = threadIdx.x; i < 4096; i += 256) lds[i] = i;
  __syncthreads();
  f16v c0={0},c1={0},c2={0},c3={0}; f4v d0={0},d1={0},d2={0},d3={0};
  float a = threadIdx.x*0.001f, b = 1.0f;
  float v0=a, v1=a+1, v2=a+2, v3=a+3; float ls = 0; int li = threadIdx.x;
  for (int it=0; it<iters; ++it) {
#pragma unroll
    for (int u=0; u<4; ++u) {
      if (KIND==0) { f16v& c = u==0?c0:u==1?c1:u==2?c2:c3; c = __builtin_amdgcn_mfma_f32_32x32x2f32(a,b,c,0,0,0); }
      else { f4v& d = u==0?d0:u==1?d1:u==2?d2:d3; d = __builtin_amdgcn_mfma_f32_16x16x4f32(a,b,d,0,0,0); }
#pragma unroll
      for (int q=0;q<V;++q){ float& v = (q&3)==0?v0:(q&3)==1?v1:(q&3)==2?v2:v3; asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(v) : "v"(b), "v"(a)); }
#pragma unroll
      for (int q=0;q<L;++q){ float t; asm volatile("ds_read_b32 %0, %1" : "=v"(t) : "v"((li*4 + q*1024 + u*256) & 16383)); asm volatile("s_waitcnt lgkmcnt(0)\n v_add_f32 %0, %0, %1" : "+v"(ls) : "v"(t)); }
    }
  }
  float s = v0+v1+v2+v3+ls; for (int r=0;r<16;++r) s += c0[r]+c1[r]+c2[r]+c3[r]; for (int r=0;r<4;++r) s += d0[r]+d1[r]+d2[r]+d3[r];
  if (s == 12345.678f) out[0] = s;
}
template<int V, int L, int KIND> void run(float* d, int wpc) {
  int blocks = 256*wpc/4, iters=4000; hipEvent_t e0,e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  k<V,L,KIND><<<blocks,256>>>(d, 10); CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0)); k<V,L,KIND><<<blocks,256>>>(d, iters); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms,e0,e1));
  double flop = (double)blocks*4*iters*4*(KIND==0?4096.0:2048.0);
  // cycles per MFMA per SIMD at 2.4GHz assumed
  double cyc = ms*1e-3*2.4e9 / ((double)iters*4*(wpc/4.0));
  printf("kind %s V=%2d L=%d waves/SIMD %d: %.1f TFLOP/s, %.1f cycles/MFMA/SIMD\n", KIND==0?"32x32x2":"16x16x4", V, L, wpc/4, flop/ms/1e9, cyc);
}
int run_part(){ float* d; CK(hipMalloc(&d, 4096));
  for (int wpc : {4, 8}) {
    run<0,0,0>(d,wpc); run<2,0,0>(d,wpc); run<4,0,0>(d,wpc); run<8,0,0>(d,wpc); run<12,0,0>(d,wpc); run<16,0,0>(d,wpc); run<24,0,0>(d,wpc);
    run<0,1,0>(d,wpc); run<0,2,0>(d,wpc); run<4,2,0>(d,wpc);
    run<0,0,1>(d,wpc); run<2,0,1>(d,wpc); run<4,0,1>(d,wpc); run<8,0,1>(d,wpc); run<0,1,1>(d,wpc); run<2,1,1>(d,wpc);
  }
  printf("done\n"); return 0; }

}  // namespace part2

namespace part3 {
// per iteration: L ds_read_b32 (consumed next iteration) + 4 independent MFMA 32x32x2
template<int L, int STRIDE> __global__ __launch_bounds__(512) void k(float* out, int iters) {
  __shared__ float lds[8192];
  for (int i = threadIdx.x; i < 8192; i += blockDim.x) lds[i] = 1.0f;
  __syncthreads();
  f16v c0={0},c1={0},c2={0},c3={0};
  float r0[8], r1[8];
  for (int q=0;q<8;++q){ r0[q]=1.f; r1[q]=1.f; }
  int lane = threadIdx.x & 63;
  const float* base = lds + (lane*STRIDE & 2047);
  for (int it=0; it<iters; it+=2) {
#pragma unroll
    for (int q=0;q<L;++q) r1[q] = base[q*64 + (it&1024)];
    __builtin_amdgcn_sched_barrier(0);
    c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(r0[0],r0[1%((L>0)?L:1)],c0,0,0,0); c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(r0[2%((L>0)?L:1)],r0[3%((L>0)?L:1)],c1,0,0,0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(r0[4%((L>0)?L:1)],r0[5%((L>0)?L:1)],c2,0,0,0); c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(r0[6%((L>0)?L:1)],r0[7%((L>0)?L:1)],c3,0,0,0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q=0;q<L;++q) r0[q] = base[q*64 + 32 + (it&1024)];
    __builtin_amdgcn_sched_barrier(0);
    c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(r1[0],r1[1%((L>0)?L:1)],c0,0,0,0); c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(r1[2%((L>0)?L:1)],r1[3%((L>0)?L:1)],c1,0,0,0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(r1[4%((L>0)?L:1)],r1[5%((L>0)?L:1)],c2,0,0,0); c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(r1[6%((L>0)?L:1)],r1[7%((L>0)?L:1)],c3,0,0,0);
    __builtin_amdgcn_sched_barrier(0);
  }
  float s = 0; for (int r=0;r<16;++r) s += c0[r]+c1[r]+c2[r]+c3[r];
  if (s == 12345.678f) out[0] = s;
}
template<int L, int STRIDE> void run(float* d, int wpb) {
  int blocks = 256, iters=8000; hipEvent_t e0,e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  k<L,STRIDE><<<blocks,wpb*64>>>(d, 16); CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0)); k<L,STRIDE><<<blocks,wpb*64>>>(d, iters); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms,e0,e1));
  double flop = (double)blocks*wpb*iters*4*4096.0;
  double cyc = ms*1e-3*2.2e9 / ((double)iters*4*(wpb/4.0));
  printf("L=%d stride=%d waves/SIMD %d: %.1f TFLOP/s, ~%.1f cycles/MFMA/SIMD\n", L, STRIDE, wpb/4, flop/ms/1e9, cyc);
}
int run_part(){ float* d; CK(hipMalloc(&d, 4096));
  for (int wpb : {4, 8}) {
    run<0,1>(d,wpb); run<1,1>(d,wpb); run<2,1>(d,wpb); run<4,1>(d,wpb); run<6,1>(d,wpb); run<8,1>(d,wpb);
    run<4,2>(d,wpb); run<8,2>(d,wpb); run<4,32>(d,wpb); 
  }
  printf("done\n"); return 0; }

}  // namespace part3

namespace part4 {
// 512 threads = 8 wavefronts, two per SIMD.  Wavefronts 0-3 ("A") run 4 independent MFMAs per
// iteration when mode & 1; wavefronts 4-7 ("B") run, per iteration, V v_fma on 4 chains, W
// ds_write_b32 and G global stores when mode & 2.  A wavefront whose bit is clear exits at once.
template<int KIND, int V, int W, int G> __global__ __launch_bounds__(512) void k(float* out, float* sink, int iters, int mode) {
  __shared__ float lds[8192];
  const int wave = threadIdx.x >> 6;
  f16v c0={0},c1={0},c2={0},c3={0}; f4v d0={0},d1={0},d2={0},d3={0};
  float a = threadIdx.x*0.001f, b = 1.0f, v0=a, v1=a+1, v2=a+2, v3=a+3;
  if (wave < 4) {
    if (!(mode & 1)) return;
    for (int it=0; it<iters; ++it) {
      if (KIND==0) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a,b,c0,0,0,0); c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a,b,c1,0,0,0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a,b,c2,0,0,0); c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(a,b,c3,0,0,0);
      } else {
        d0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a,b,d0,0,0,0); d1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a,b,d1,0,0,0);
        d2 = __builtin_amdgcn_mfma_f32_16x16x4f32(a,b,d2,0,0,0); d3 = __builtin_amdgcn_mfma_f32_16x16x4f32(a,b,d3,0,0,0);
      }
    }
  } else {
    if (!(mode & 2)) return;
    float* g = sink + (size_t)blockIdx.x * 512 * 8 + threadIdx.x;
    for (int it=0; it<iters; ++it) {
#pragma unroll
      for (int q=0;q<V;++q){ float& v = (q&3)==0?v0:(q&3)==1?v1:(q&3)==2?v2:v3; asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(v) : "v"(b), "v"(a)); }
#pragma unroll
      for (int q=0;q<W;++q) asm volatile("ds_write_b32 %0, %1" :: "v"((threadIdx.x*4 + q*2048) & 32767), "v"(v0) : "memory");
#pragma unroll
      for (int q=0;q<G;++q) g[q*512] = v1;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  float s = v0+v1+v2+v3+lds[threadIdx.x]; for (int r=0;r<16;++r) s += c0[r]+c1[r]+c2[r]+c3[r]; for (int r=0;r<4;++r) s += d0[r]+d1[r]+d2[r]+d3[r];
  if (s == 12345.678f) out[0] = s;
}
template<int KIND, int V, int W, int G> void run(float* d, float* sink) {
  const int blocks = 256, iters = 2000; hipEvent_t e0,e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  float ms[4] = {0,0,0,0};
  for (int mode = 1; mode <= 3; ++mode) {
    k<KIND,V,W,G><<<blocks,512>>>(d, sink, 10, mode); CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0)); k<KIND,V,W,G><<<blocks,512>>>(d, sink, iters, mode); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    CK(hipEventElapsedTime(&ms[mode],e0,e1));
  }
  printf("%s x4/iter | other wave per iter: %2d v_fma %2d ds_write %d global stores | MFMA alone %.3f ms, other alone %.3f ms, both %.3f ms (sum %.3f, max %.3f)\n",
         KIND==0?"32x32x2":"16x16x4", V, W, G, ms[1], ms[2], ms[3], ms[1]+ms[2], ms[1]>ms[2]?ms[1]:ms[2]);
}
int run_part(){ float *d, *sink; CK(hipMalloc(&d, 4096)); CK(hipMalloc(&sink, (size_t)256*512*8*4));
  run<0,16,0,0>(d,sink); run<0,32,0,0>(d,sink); run<0,64,0,0>(d,sink);
  run<1,16,0,0>(d,sink); run<1,32,0,0>(d,sink);
  run<0,0,16,0>(d,sink); run<0,0,32,0>(d,sink);
  run<0,0,0,4>(d,sink); run<0,0,0,8>(d,sink);
  run<0,16,8,2>(d,sink);
  printf("done\n"); return 0; }
}  // namespace part4

int main(int argc, char** argv)
{
    const int only = argc > 1 ? atoi(argv[1]) : 0;   // 0 = every part
    if (!only || only == 1) part1::run_part();
    if (!only || only == 2) part2::run_part();
    if (!only || only == 3) part3::run_part();
    if (!only || only == 4) part4::run_part();
    return 0;
}
