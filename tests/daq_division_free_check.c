// Host check of the arithmetic the DAQ kernels use in place of a division per element (Step 3, eq. (4)):
// for every code range qmax = 2^(b-1) - 1, b = 2..8, every fp16 clipping threshold tau (the block maximum, or the
// percentile of the clipped form) and every fp16 value not above it (larger values are clipped to tau itself), the
// code taken from fma(x, fl(1/alpha), 1.5*2^23), alpha = fl(tau / qmax), equals clamp(rint(fl(x/alpha))) whenever
// |fma(x, fl(1/alpha), -r)| < 0.5 - 2^-15, i.e. whenever the kernel does not fall back to the division.
// Prints the counts per qmax; exit status 1 on any mismatch.
#include <stdio.h>
#include <stdint.h>
#include <string.h>
#include <math.h>
static float h2f(uint16_t h){ uint32_t s=(h>>15)&1,e=(h>>10)&31,m=h&1023; float f; if(e==0) f=ldexpf((float)m,-24); else if(e==31) f=m?NAN:INFINITY; else f=ldexpf((float)(m+1024),(int)e-25); return s?-f:f; }
int main(void){
  const float MAGIC=12582912.0f, THR=0.5f-0.000030517578125f;
  int fail=0;
  for (int b=8; b>=2; --b){
    const float qmax=(float)((1<<(b-1))-1);
    unsigned long long total=0, slow=0, bad=0, badrange=0;
    #pragma omp parallel for schedule(dynamic,64) reduction(+:total,slow,bad,badrange)
    for (int am=1; am<=0x7bff; ++am){
      float tau=h2f((uint16_t)am); float alpha=tau/qmax; float rcp=1.0f/alpha;
      for (int xb=0; xb<=am; ++xb){
        float x=h2f((uint16_t)xb);
        float t=x/alpha; float r0=rintf(t); if(r0>qmax) r0=qmax; if(r0<-qmax) r0=-qmax; int c0=(int)r0;
        float y=fmaf(x,rcp,MAGIC); float r=y-MAGIC; float d=fmaf(x,rcp,-r);
        uint32_t yb; memcpy(&yb,&y,4); int c1=(int)(int8_t)(yb&0xff);
        total++;
        if(!(fabsf(d)<THR)) { slow++; continue; }
        if(c1!=c0) bad++;
        if(r>qmax||r<-qmax) badrange++;
        // negative x
        float yn=fmaf(-x,rcp,MAGIC); memcpy(&yb,&yn,4); int c2=(int)(int8_t)(yb&0xff);
        if(c2!=-c0) bad++;
      }
    }
    printf("qmax %d pairs %llu slow %llu (%.3g) mismatches %llu out-of-range %llu\n", (int)qmax, total, slow, (double)slow/total, bad, badrange);
    if (bad||badrange) fail=1;
  }
  return fail;
}
