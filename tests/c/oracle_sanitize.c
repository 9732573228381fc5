/* Host-only driver for AddressSanitizer / UBSan: every oracle schedule for p = 1..70 and
 * Allgatherv geometries for p = 1..40, each checked against the definition. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
int oracle_allgather(int algo, int p, size_t B, const void *send, void *recv, int max_steps, int32_t *step_info, int64_t *sent, int32_t *trace, size_t cap, size_t *len);
int oracle_allgatherv(int algo, int p, const size_t *counts, const size_t *displs, size_t row, const void *send, void *recv, int max_steps, int32_t *si, int64_t *sent, int32_t *trace, size_t cap, size_t *len);
int main(void){
  int bad=0;
  for(int algo=0; algo<4; algo++) for(int p=1;p<=70;p++){ size_t B=3; 
    unsigned char *send=malloc(p*B), *recv=malloc((size_t)p*p*B); for(size_t i=0;i<p*B;i++) send[i]=(unsigned char)(i*7+1); memset(recv,0xA5,(size_t)p*p*B);
    int32_t *trace=malloc((size_t)p*p*5*4); size_t n=0; int32_t si[3*80]; int64_t *sent=malloc(p*8);
    int rc=oracle_allgather(algo,p,B,send,recv,-1,si,sent,trace,(size_t)p*p,&n);
    if(algo==2 && (p&(p-1))) { if(rc!=-8) bad++; } else { if(rc) bad++; for(int r=0;r<p;r++) if(memcmp(recv+(size_t)r*p*B, send, p*B)) bad++; }
    free(send);free(recv);free(trace);free(sent);
  }
  for(int p=1;p<=40;p++){ size_t counts[40], displs[40], at=0; for(int k=0;k<p;k++){ counts[k]=(k*5+p)%9; displs[k]=at+1; at+=counts[k]+1; } size_t row=at+2;
    unsigned char *send=malloc(row), *recv=malloc(p*row); for(size_t i=0;i<row;i++) send[i]=(unsigned char)(i*3+2); memset(recv,0xA5,p*row);
    int rc=oracle_allgatherv(0,p,counts,displs,row,send,recv,-1,NULL,NULL,NULL,0,NULL); if(rc) bad++;
    for(int r=0;r<p;r++) for(int k=0;k<p;k++) if(memcmp(recv+r*row+displs[k], send+displs[k], counts[k])) bad++;
    free(send);free(recv);
  }
  printf("bad=%d\n",bad); return bad!=0;
}
