// Drives the sequencer's C ABI under sanitizers with long random event streams: swap-outs,
// requests of swaps and small transfers, writes into kept chunks, stray syncs.  Prints how many
// actions came out; the sanitizers do the checking.  Test infrastructure.
#include <cstdio>
#include <cstdint>
#include <vector>
#include "pgcm_seq.h"
static uint64_t st=88172645463325252ull; static uint64_t rnd(){ st^=st<<13; st^=st>>7; st^=st<<17; return st; }
int main(){
  uint64_t total=0;
  for(int trial=0; trial<300; ++trial){
    pgcm_seq_t* s=nullptr;
    if(pgcm_seq_create(rnd()%100, 1+rnd()%6, rnd()%3, 128*1024, 1+rnd()%64, &s)!=0) return 1;
    std::vector<pgcm_seq_action> acts(7);
    for(int e=0;e<400;++e){
      uint64_t r=rnd()%100; uint64_t addr=0x1000000+(rnd()%12)*(1<<20); uint64_t len=(rnd()%3==0)? 200000 : (1<<20);
      if(r<45) pgcm_seq_request(s,addr,len); else if(r<65) pgcm_seq_swap_out(s,addr,len);
      else if(r<75) pgcm_seq_notify_write(s,addr+rnd()%len,1+rnd()%4096); else if(r<85) pgcm_seq_request(s,0x7000000+rnd()%1000*64,1+rnd()%8000);
      else pgcm_seq_sync(s);
      size_t n; while((n=pgcm_seq_take_actions(s,acts.data(),acts.size()))>0) total+=n;
    }
    pgcm_seq_sync(s);
    size_t n; while((n=pgcm_seq_take_actions(s,acts.data(),acts.size()))>0) total+=n;
    pgcm_seq_destroy(s);
  }
  uint8_t iv0[12]={255,255,255,255,255,255,255,255,255,255,255,250}, out[12];
  pgcm_seq_iv_bytes(iv0, 10, out);
  printf("actions %llu, iv wrap byte %u\n",(unsigned long long)total,out[11]);
  return 0;
}
