/* A caller of the C ABI written in C: compiled by tests/test_abi_host.py with gcc against include/fs.h and
 * the library (the header must be plain C).  It describes one fusion group -- softmax over the rows of a
 * [64, 256] fp32 tensor, as XLA-style ops -- asks for a plan, prints what the plan is, and checks the error
 * path with a malformed list.  No GPU is touched: planning is host work. */
#include <stdio.h>
#include <string.h>
#include "fs.h"

static fs_op_desc op(int32_t kind, int32_t rank, int64_t d0, int64_t d1, int32_t a, int32_t b, int32_t axis, double attr) {
  fs_op_desc o;
  memset(&o, 0, sizeof o);
  o.kind = kind; o.dtype = FS_F32; o.rank = rank; o.axis = axis;
  o.shape[0] = d0; o.shape[1] = d1;
  o.operand[0] = a; o.operand[1] = b; o.operand[2] = -1;
  o.attr = attr;
  return o;
}

int main(void) {
  const int64_t R = 64, C = 256;
  fs_op_desc ops[9];
  ops[0] = op(FS_PARAMETER, 2, R, C, -1, -1, 0, 0.0);      /* x                         */
  ops[1] = op(FS_REDUCE_MAX, 1, R, 0, 0, -1, 1, 0.0);      /* m = max over the row      */
  ops[2] = op(FS_BROADCAST, 2, R, C, 1, -1, 0, 0.0);       /* m back to [R, C]          */
  ops[3] = op(FS_SUBTRACT, 2, R, C, 0, 2, 0, 0.0);         /* x - m                     */
  ops[4] = op(FS_EXP, 2, R, C, 3, -1, 0, 0.0);             /* e = exp(x - m)            */
  ops[5] = op(FS_REDUCE_SUM, 1, R, 0, 4, -1, 1, 0.0);      /* s = sum over the row      */
  ops[6] = op(FS_BROADCAST, 2, R, C, 5, -1, 0, 0.0);
  ops[7] = op(FS_DIVIDE, 2, R, C, 4, 6, 0, 0.0);           /* e / s                     */
  ops[8] = op(FS_OUTPUT, 2, R, C, 7, -1, 0, 0.0);
  fs_plan* plan = NULL;
  fs_status st = fs_plan_create(ops, 9, NULL, &plan);
  if (st != FS_OK || !plan) { printf("create failed: %d %s\n", (int)st, fs_last_error()); return 1; }
  int32_t schedule = -1, n_kernels = -1;
  int64_t lds = -1, ws = -1, algo = -1, moved = -1;
  if (fs_plan_info(plan, &schedule, &n_kernels, &lds, &ws, &algo, &moved) != FS_OK) return 2;
  printf("schedule=%d kernels=%d lds=%lld workspace=%lld algorithmic_bytes=%lld\n", (int)schedule, (int)n_kernels,
         (long long)lds, (long long)ws, (long long)algo);
  printf("template: %s\n", fs_plan_describe(plan));
  if (schedule != FS_SCHED_ROW || n_kernels != 1 || algo != 2 * R * C * 4) return 3;
  if (fs_destroy(plan) != FS_OK) return 4;
  /* an operand that points forward: refused with a message, no plan handed out */
  ops[3].operand[1] = 7;
  plan = NULL;
  st = fs_plan_create(ops, 9, NULL, &plan);
  if (st != FS_ERR_INVALID || plan != NULL || !fs_last_error()[0]) return 5;
  printf("refused: %s\n", fs_last_error());
  return 0;
}
