// Host-only fuzz driver for the selector entry points; built with the address and
// undefined-behaviour sanitizers by tests/test_host_sanitizers.py (no GPU code involved).
#include "gemm.h"
#include <cstdio>
#include <cstdlib>
int main(){ gemm_cfg c; gemm_prediction p; long n=0; unsigned s=1;
  for(int it=0; it<3000; ++it){ s=s*1664525u+1013904223u; long M=1+(s>>8)%16384; s=s*1664525u+1013904223u; long N=16*(1+(s>>8)%1024); s=s*1664525u+1013904223u; long K=16*(1+(s>>8)%1024); int dt=it&1;
    if(gemm_select(M,N,K,dt,&c)!=0){printf("select failed %ld %ld %ld\n",M,N,K);return 1;} if(gemm_predict(&c,&p)!=0) return 2; n+=c.kernel_id;
    for(int i=0;i<gemm_cfg_count(dt);i+=7){ gemm_cfg d; int rc=gemm_cfg_at(i,M,N,K,dt,&d); if(rc!=0&&rc!=GEMM_ERR_CFG_ILLEGAL) return 3; } }
  gemm_hw h; gemm_hw_get(&h); h.n_cu=304; h.n_xcd=8; gemm_hw_set(&h); gemm_select(4096,4096,4096,0,&c); gemm_hw_reset();
  printf("ok %ld\n",n); return 0; }
