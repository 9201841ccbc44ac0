/* Test infrastructure: a stand-in for the profiler's marker library.  It has the three entry points
 * the runtime looks up and appends every call to the file named by ROCTX_RECORD. */
#include <stdio.h>
#include <stdlib.h>

static void record(const char* kind, const char* msg) {
  const char* path = getenv("ROCTX_RECORD");
  if (!path) return;
  FILE* f = fopen(path, "a");
  if (!f) return;
  fprintf(f, "%s %s\n", kind, msg ? msg : "");
  fclose(f);
}
int roctxRangePushA(const char* msg) { record("push", msg); return 0; }
int roctxRangePop(void) { record("pop", ""); return 0; }
void roctxMarkA(const char* msg) { record("mark", msg); }
