// In-bounds probe of builtin lane layouts on gfx950: mfma 32x32x16 bf16, 16x16x32 bf16, ds_read_tr16_b64.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#include <vector>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

__device__ __bf16 tobf(float f){ unsigned u=__float_as_uint(f); unsigned short s=u>>16; __bf16 r; __builtin_memcpy(&r,&s,2); return r; }

__global__ void k_mfma32(const float* A, const float* B, float* Craw){ // A[32][16], B[16][32]
  int l=threadIdx.x; int i=l%32, g=l/32;
  bf16x8 a,b;
  for(int j=0;j<8;j++){ a[j]=tobf(A[i*16+8*g+j]); b[j]=tobf(B[(8*g+j)*32+i]); }
  f32x16 c={0};
  c=__builtin_amdgcn_mfma_f32_32x32x16_bf16(a,b,c,0,0,0);
  for(int v=0;v<16;v++) Craw[l*16+v]=c[v];
}
__global__ void k_mfma16(const float* A, const float* B, float* Craw){ // A[16][32], B[32][16]
  int l=threadIdx.x; int i=l%16, g=l/16;
  bf16x8 a,b;
  for(int j=0;j<8;j++){ a[j]=tobf(A[i*32+8*g+j]); b[j]=tobf(B[(8*g+j)*16+i]); }
  f32x4 c={0};
  c=__builtin_amdgcn_mfma_f32_16x16x32_bf16(a,b,c,0,0,0);
  for(int v=0;v<4;v++) Craw[l*4+v]=c[v];
}
__global__ void k_tr(unsigned short* out){
  __shared__ unsigned short lds[1024];
  int l=threadIdx.x;
  for(int i=l;i<1024;i+=64) lds[i]=i;
  __syncthreads();
  s16x4 v=__builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(lds+4*l));
  for(int j=0;j<4;j++) out[l*4+j]=v[j];
}
int main(){
  float hA[512],hB[512]; for(int i=0;i<512;i++){hA[i]=(float)((i*7)%11-5); hB[i]=(float)((i*5)%13-6);}
  float *dA,*dB,*dC; hipMalloc(&dA,2048);hipMalloc(&dB,2048);hipMalloc(&dC,4096);
  hipMemcpy(dA,hA,2048,hipMemcpyHostToDevice);hipMemcpy(dB,hB,2048,hipMemcpyHostToDevice);
  std::vector<float> C(1024);
  k_mfma32<<<1,64>>>(dA,dB,dC); hipMemcpy(C.data(),dC,4096,hipMemcpyDeviceToHost);
  { int bad=0; for(int l=0;l<64;l++)for(int v=0;v<16;v++){ int col=l%32; int row=(v/4)*8+(l/32)*4+(v%4); float r=0; for(int k=0;k<16;k++) r+=hA[row*16+k]*hB[k*32+col]; if(r!=C[l*16+v]) bad++; }
    printf("mfma32x32x16 hypothesized layout mismatches: %d\n",bad); }
  k_mfma16<<<1,64>>>(dA,dB,dC); hipMemcpy(C.data(),dC,1024,hipMemcpyDeviceToHost);
  { int bad=0; for(int l=0;l<64;l++)for(int v=0;v<4;v++){ int col=l%16; int row=(l/16)*4+v; float r=0; for(int k=0;k<32;k++) r+=hA[row*32+k]*hB[k*16+col]; if(r!=C[l*4+v]) bad++; }
    printf("mfma16x16x32 hypothesized layout mismatches: %d\n",bad); }
  unsigned short* dO; hipMalloc(&dO,512); unsigned short hO[256];
  k_tr<<<1,64>>>(dO); hipMemcpy(hO,dO,512,hipMemcpyDeviceToHost);
  for(int l=0;l<64;l++) printf("tr lane %2d: %4d %4d %4d %4d\n",l,hO[l*4],hO[l*4+1],hO[l*4+2],hO[l*4+3]);
  hipError_t e=hipDeviceSynchronize(); printf("status %s\n",hipGetErrorString(e));
  return 0;
}
