// Measures the LDS read bandwidth of a compute unit (MI355X, gfx950): conflict-free streams of
// ds_read_b32 / b64 / b128, four reads in flight per wavefront, issued by inline asm so that the
// arithmetic beside a read is one xor.  It backs the LDS ceiling that bench.py prices the scan
// kernel against; it is not part of libspd.so.
//
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o lds_bandwidth paper_2104_06357_amd/microbench/lds_bandwidth.hip && ./lds_bandwidth
//
// Every address is masked into the 64 KB array: no access leaves it.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("err %s line %d\n",hipGetErrorString(e),__LINE__); exit(1);} }while(0)
typedef unsigned u4 __attribute__((ext_vector_type(4)));
typedef unsigned u2 __attribute__((ext_vector_type(2)));
template <int WIDTH, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k(unsigned* out, int iters){
  __shared__ unsigned s[16384];
  for(int i=threadIdx.x;i<16384;i+=BLOCK) s[i]=i*7;
  __syncthreads();
  unsigned acc=0;
  unsigned base = (unsigned)(size_t)s;             // LDS byte address of the array
  unsigned lane_off = threadIdx.x * WIDTH;         // a wavefront reads 64 consecutive items
  for(int it=0; it<iters; ++it){
    unsigned a0 = base + ((lane_off + it*64*WIDTH) & 0xFFFF & ~(WIDTH-1));
    unsigned a1 = base + ((lane_off + it*64*WIDTH + 16384) & 0xFFFF & ~(WIDTH-1));
    unsigned a2 = base + ((lane_off + it*64*WIDTH + 32768) & 0xFFFF & ~(WIDTH-1));
    unsigned a3 = base + ((lane_off + it*64*WIDTH + 49152) & 0xFFFF & ~(WIDTH-1));
    if constexpr (WIDTH==16){ u4 v0,v1,v2,v3;
      asm volatile("ds_read_b128 %0, %4\n ds_read_b128 %1, %5\n ds_read_b128 %2, %6\n ds_read_b128 %3, %7\n s_waitcnt lgkmcnt(0)" : "=&v"(v0),"=&v"(v1),"=&v"(v2),"=&v"(v3) : "v"(a0),"v"(a1),"v"(a2),"v"(a3) : "memory");
      acc ^= v0.x ^ v1.y; acc ^= v2.z ^ v3.w; }
    else if constexpr (WIDTH==8){ u2 v0,v1,v2,v3;
      asm volatile("ds_read_b64 %0, %4\n ds_read_b64 %1, %5\n ds_read_b64 %2, %6\n ds_read_b64 %3, %7\n s_waitcnt lgkmcnt(0)" : "=&v"(v0),"=&v"(v1),"=&v"(v2),"=&v"(v3) : "v"(a0),"v"(a1),"v"(a2),"v"(a3) : "memory");
      acc ^= v0.x ^ v1.y; acc ^= v2.x ^ v3.y; }
    else { unsigned v0,v1,v2,v3;
      asm volatile("ds_read_b32 %0, %4\n ds_read_b32 %1, %5\n ds_read_b32 %2, %6\n ds_read_b32 %3, %7\n s_waitcnt lgkmcnt(0)" : "=&v"(v0),"=&v"(v1),"=&v"(v2),"=&v"(v3) : "v"(a0),"v"(a1),"v"(a2),"v"(a3) : "memory");
      acc ^= v0 ^ v1; acc ^= v2 ^ v3; }
  }
  out[blockIdx.x*BLOCK+threadIdx.x]=acc;
}
template <int WIDTH, int BLOCK> void run(int grid){
  unsigned* out; CK(hipMalloc(&out, (size_t)grid*BLOCK*4));
  int iters=4000;
  hipEvent_t a,b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  k<WIDTH,BLOCK><<<grid,BLOCK>>>(out,10); CK(hipDeviceSynchronize());
  CK(hipEventRecord(a)); k<WIDTH,BLOCK><<<grid,BLOCK>>>(out,iters); CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
  float ms; CK(hipEventElapsedTime(&ms,a,b));
  double bytes=(double)grid*BLOCK*iters*4.0*WIDTH;
  printf("ds_read_b%d block %d grid %d: %.3f ms, %.1f TB/s, %.1f B/clk/CU (256 CUs x 2.4 GHz)\n", WIDTH*8, BLOCK, grid, ms, bytes/ms/1e9, bytes/(ms*1e-3)/256/2.4e9);
  fflush(stdout);
  CK(hipFree(out));
}
int main(){
  run<4,1024>(512); run<8,1024>(512); run<16,1024>(512);
  run<4,512>(512); run<8,512>(512); run<16,512>(512);
  run<16,1024>(256);
  return 0;
}
