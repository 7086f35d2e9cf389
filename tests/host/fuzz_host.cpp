// Random inputs through the library's host-only code (plan building with its tile table,
// shares, sampler partition), meant to be built with -fsanitize=address,undefined.
// usage: fuzz_host [iterations]
#include <cstdio>
#include <cstdlib>
#include <cstdarg>
#include <random>
#include <vector>
#include "kt_internal.h"
void kt_set_error(const char *fmt, ...) { (void)fmt; }
int main(int argc, char **argv) {
  const int iters = argc > 1 ? atoi(argv[1]) : 20000;
  std::mt19937_64 rng(1);
  long plans=0, tiles=0;
  for (int it=0; it<iters; ++it) {
    int T = rng()%40; std::vector<int64_t> n(T);
    for (auto &x: n) { int m=rng()%4; x = m==0? rng()%8 : m==1? rng()%3000 : m==2? rng()%40000 : (rng()%5==0? 0 : rng()%200); }
    kt_dtype dt = (rng()&1)? KT_F32: KT_BF16; int es = dt==KT_F32?4:2;
    int align = es << (rng()%14); if (align>16384) align=16384;
    int64_t caps[]={0,64,1000,4096,65536,200000}; int64_t cap=caps[rng()%6];
    KtHostPlan hp; const char* msg="";
    kt_status st = kt_build_host_plan(n.data(), T, dt, cap, align, hp, &msg);
    if (st!=KT_OK) { printf("unexpected %d %s\n", st, msg); return 1; }
    plans++; tiles+=hp.tiles.size();
    // replay kernel-side assumptions
    for (auto &tl: hp.tiles) {
      int b=tl.bucket; int first=hp.b_first[b], last=first+hp.b_count[b]-1;
      int cnt = tl.nt==0?1:tl.nt;
      if (tl.t0<first || tl.t0+cnt-1>last) { printf("tile range\n"); return 1; }
    }
  }
  for (int it=0; it<iters; ++it) {
    int K=1+rng()%16; double thr[64]; for(int k=0;k<K;++k) thr[k]=(1+rng()%1000)/100.0;
    int64_t B=rng()%100000; int64_t sh[64]; float w[64];
    if (kt_plan_shares(thr,K,B,sh,B>0?w:nullptr)!=KT_OK) { printf("shares\n"); return 1; }
    int64_t s=0; for(int k=0;k<K;++k) s+=sh[k]; if (s!=B) { printf("sum\n"); return 1; }
    if (B>0 && it%10==0) {
      int64_t N=rng()%5000; int rank=rng()%K; int64_t cnt;
      if (kt_sampler_epoch_size(N,B,sh,K,rank,rng()&1,&cnt)!=KT_OK) { printf("ssize\n"); return 1; }
      std::vector<int64_t> out((size_t)(cnt>0?cnt:1));
      int dl=rng()&1; kt_sampler_epoch_size(N,B,sh,K,rank,dl,&cnt); out.resize((size_t)(cnt>0?cnt:1));
      if (kt_sampler_epoch(N,B,sh,K,rng(),rng()%100,rng()&1,rank,dl,out.data(),cnt,nullptr)!=KT_OK) { printf("sampler\n"); return 1; }
      for (int64_t i=0;i<cnt;++i) if (out[i]<0||out[i]>=N) { printf("idx\n"); return 1; }
    }
  }
  printf("ok plans=%ld tiles=%ld\n", plans, tiles);
  return 0;
}
