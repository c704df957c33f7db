// in-bounds probe: where does buffer_load_dwordx4 ... lds put each lane's 16 bytes?
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
__global__ void k(const unsigned* src, unsigned* out){
  __shared__ unsigned lds[1024];
  for (int i=threadIdx.x;i<1024;i+=64) lds[i]=0xdeadbeef;
  __syncthreads();
  __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void*)src, 0, 4096, 0x00020000);
  // lane L fetches global granule (63-L) so that the LDS placement shows the lane index
  unsigned voff = (63 - threadIdx.x) * 16;
  if (threadIdx.x == 5) voff = 0x80000000u;   // out of range lane: expect zeros
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void*)&lds[64], 16, voff, 0, 0, 0);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  for (int i=threadIdx.x;i<1024;i+=64) out[i]=lds[i];
}
int main(){
  unsigned h[1024]; for(int i=0;i<1024;i++) h[i]=i;
  unsigned *s,*o; hipMalloc(&s,4096); hipMalloc(&o,4096); hipMemcpy(s,h,4096,hipMemcpyHostToDevice);
  k<<<1,64>>>(s,o); hipMemcpy(h,o,4096,hipMemcpyDeviceToHost);
  for(int i=0;i<384;i+=4) printf("lds[%3d..]: %08x %08x %08x %08x\n",i,h[i],h[i+1],h[i+2],h[i+3]);
  printf("%s\n", hipGetErrorString(hipDeviceSynchronize()));
}
