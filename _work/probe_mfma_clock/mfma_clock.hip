// Stand-alone probe (not part of the library): what does the dense bf16 MFMA peak depend on?
// A register-only MFMA loop (v_mfma_f32_32x32x16_bf16, independent accumulators, 256 workgroups) is timed with
// operands of zeros, ones and random bf16 values; the shader clock during the loop is read from the cycle
// counter against the constant 100 MHz clock.  On MI355X the rate follows the clock, and the clock follows the
// operand data (power limit): this is the ceiling any real-data bf16 GEMM kernel has on this part.
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -o mfma_clock mfma_clock.hip && ./mfma_clock
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
template<int NA, int NB, int NT, int BAR>
__global__ void __launch_bounds__(NT) k(const uint4* in, float* out, long long* clk, int iters){
  f32x16 acc[NA][NB];
  for(int i=0;i<NA;i++) for(int j=0;j<NB;j++) for(int e=0;e<16;e++) acc[i][j][e]=0.f;
  uint4 fa[NA], fb[NB];
  for(int i=0;i<NA;i++) fa[i]=in[(threadIdx.x*7+i*64)&4095];
  for(int j=0;j<NB;j++) fb[j]=in[(threadIdx.x*5+j*64+2048)&4095];
  long long t0 = clock64();
  long long w0 = wall_clock64();
  for(int it=0; it<iters; ++it){
#pragma unroll
    for(int i=0;i<NA;i++)
#pragma unroll
      for(int j=0;j<NB;j++) acc[i][j]=__builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8,fa[i]),__builtin_bit_cast(bf16x8,fb[j]),acc[i][j],0,0,0);
    if (BAR) __builtin_amdgcn_s_barrier();
  }
  long long t1 = clock64();
  long long w1 = wall_clock64();
  float s=0; for(int i=0;i<NA;i++) for(int j=0;j<NB;j++) for(int e=0;e<16;e++) s+=acc[i][j][e];
  if(s==12345.f) out[0]=s;
  if (threadIdx.x==0 && blockIdx.x==0) { clk[0]=t1-t0; clk[1]=w1-w0; }
}
template<typename F> double timeit(F f){
  hipEvent_t e0,e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  f(); CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0)); f(); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms,e0,e1)); return ms;
}
int main(){
  float* out; CK(hipMalloc(&out,4));
  long long* clk; CK(hipMalloc(&clk,16));
  uint4* in; CK(hipMalloc(&in, 4096*16));
  unsigned* h = (unsigned*)malloc(4096*16);
  int it2=20000;
  const char* names[3]={"zeros","ones","random"};
  for (int d=0; d<3; ++d) {
    for (int i=0;i<4096*4;i++) { if(d==0) h[i]=0; else if(d==1) h[i]=0x3f803f80; else { unsigned a = (rand()&0xffff), b=(rand()&0xffff); a = (a & 0x807f) | ((120 + (rand()%12))<<7); b = (b & 0x807f) | ((120 + (rand()%12))<<7); h[i] = a | (b<<16);} }
    CK(hipMemcpy(in,h,4096*16,hipMemcpyHostToDevice));
#define RUN(NA,NB,NT,BAR,label) { double ms=timeit([&]{ k<NA,NB,NT,BAR><<<256,NT>>>(in,out,clk,it2); }); long long hc[2]; CK(hipMemcpy(hc,clk,16,hipMemcpyDeviceToHost)); double fl=256.0*(NT/64)*it2*(NA*NB)*32768.0; printf("%-7s %-34s: %.1f TFLOP/s, %.2f ms, shader clk %.0f MHz\n", names[d], label, fl/ms/1e9, ms, (double)hc[0]/((double)hc[1]/100.0)); }
    RUN(2,4,512,0,"8 waves 2x4, no barrier");
    RUN(2,4,512,1,"8 waves 2x4, barrier / 8 mfma");
    RUN(4,4,256,0,"4 waves 4x4, no barrier");
    RUN(4,4,256,1,"4 waves 4x4, barrier / 16 mfma");
  }
  printf("done\n"); return 0;
}
