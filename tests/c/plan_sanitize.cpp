// Host-only driver for AddressSanitizer / UBSan: builds every schedule's tables for p = 1..300
// through the C ABI and walks all of them.
#include <cstdio>
#include "sparbit.h"
int main(){ long total=0; for(int algo=0;algo<5;algo++) for(int p=1;p<=300;p++){ sparbit_plan_t* pl=nullptr; int rc=sparbit_plan_create(p,algo,&pl); if(rc){ if(!(algo==2 && (p&(p-1)))) {printf("rc %d algo %d p %d\n",rc,algo,p); return 1;} continue;} int n=sparbit_plan_num_steps(pl); for(int s=0;s<n;s++){ sparbit_step_t st; if(sparbit_plan_step(pl,s,&st)) return 1; for(int r=0;r<p;r++){ total+=st.dst[r]+st.src[r]; for(int j=0;j<st.nblocks;j++) total+=st.send_slot[(size_t)r*st.nblocks+j]+st.recv_slot[(size_t)r*st.nblocks+j]; } } sparbit_plan_destroy(pl);} printf("ok %ld\n",total); return 0; }
