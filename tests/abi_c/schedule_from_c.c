/* The header is plain C: this file is compiled with a C compiler, linked against libhanayo.so and run
 * by tests/test_abi.py.  It asks for rank 0's task list of (P, W, M) = (4, 2, 8) and its stash plan and
 * prints them, one task per line, for the test to compare with the oracle. */
#include <stdio.h>
#include <stdlib.h>

#include "hanayo.h"

int main(void) {
  size_t n = 0;
  int rc = hanayo_schedule(4, 2, 8, 0, NULL, 0, &n);
  if (rc != HANAYO_EBUFSIZE || n != 64) {
    fprintf(stderr, "query: rc %d n %zu\n", rc, n);
    return 1;
  }
  hanayo_task* list = (hanayo_task*)malloc(n * sizeof(hanayo_task));
  int32_t* slot = (int32_t*)malloc(n * sizeof(int32_t));
  int per_chunk[4], peak = 0;
  rc = hanayo_schedule(4, 2, 8, 0, list, n, &n);
  if (rc == HANAYO_OK) rc = hanayo_stash_plan(list, n, 2, &peak, per_chunk, slot);
  if (rc != HANAYO_OK) {
    fprintf(stderr, "%s: %s\n", hanayo_strerror(rc), hanayo_last_error());
    return 1;
  }
  printf("peak %d\n", peak);
  for (size_t i = 0; i < n; ++i)
    printf("%c %u %u %u %d\n", list[i].kind == HANAYO_F ? 'F' : 'B', list[i].mb, (unsigned)list[i].chunk, list[i].stage,
           (int)slot[i]);
  /* the argument blocks are complete types in C */
  hanayo_exec_args ea;
  hanayo_pipeline_args pa;
  hanayo_ends_args en;
  hanayo_adam ad;
  (void)ea; (void)pa; (void)en; (void)ad;
  free(list);
  free(slot);
  return 0;
}
