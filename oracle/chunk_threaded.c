/*
 * A multi-core CPU baseline built on the oracle, for the benchmark's reported CPU figure.
 * TEST INFRASTRUCTURE ONLY, like the rest of this folder.
 *
 * It is the same definition executed with more cores: one serial pass over the arrivals
 * decides, in arrival order, which record of every sequence number is applied (the bitmap
 * step has to see the arrivals in order); the chosen records are then dealt to threads,
 * and every thread applies its records by calling orc_apply() itself, one record per call,
 * with a private, all-clear seen[] array.  Records with different sequence numbers touch
 * disjoint memory (the call's precondition), so the order among threads cannot matter and
 * the result equals orc_apply() over the whole call bit for bit -- a CPU test holds it to that.
 */
#define _POSIX_C_SOURCE 200809L
#include <pthread.h>
#include <stdlib.h>
#include <string.h>

#include "chunk_oracle.h"

typedef struct {
  void* acc; uint64_t acc_bytes; void* out_stage; uint64_t out_bytes;
  const void* recv_stage; uint64_t recv_bytes; const orc_desc* descs;
  const uint64_t* chosen; uint64_t begin, end; uint64_t n_bits; int dtype, op;
  int64_t status;
} job;

static void* worker(void* p) {
  job* j = (job*)p;
  uint8_t* mine = (uint8_t*)calloc(j->n_bits ? j->n_bits : 1, 1);
  if (!mine) { j->status = ORC_E_ARG; return NULL; }
  for (uint64_t i = j->begin; i < j->end; ++i) {
    int64_t rc = orc_apply(j->acc, j->acc_bytes, j->out_stage, j->out_bytes, j->recv_stage, j->recv_bytes,
                           &j->descs[j->chosen[i]], 1, mine, j->n_bits, j->dtype, j->op);
    if (rc != 1) { j->status = rc < 0 ? rc : ORC_E_ARG; break; }
  }
  free(mine);
  return NULL;
}

int64_t orc_apply_threaded(void* acc, uint64_t acc_bytes, void* out_stage, uint64_t out_bytes,
                           const void* recv_stage, uint64_t recv_bytes, const orc_desc* descs,
                           uint64_t n_descs, uint8_t* seen, uint64_t n_bits, int dtype, int op,
                           int n_threads) {
  if (n_threads < 1 || n_threads > 256) return ORC_E_ARG;
  if (n_descs == 0) return 0;
  if (!descs || !seen) return ORC_E_ARG;
  uint64_t* chosen = (uint64_t*)malloc(sizeof(uint64_t) * n_descs);
  if (!chosen) return ORC_E_ARG;
  uint64_t n_chosen = 0;
  for (uint64_t k = 0; k < n_descs; ++k) { /* arrival order */
    if (descs[k].seq >= n_bits) { free(chosen); return ORC_E_SEQ; }
    if (seen[descs[k].seq]) continue;
    seen[descs[k].seq] = 1;
    chosen[n_chosen++] = k;
  }
  job jobs[256];
  pthread_t tid[256];
  int started = 0;
  int64_t status = (int64_t)n_chosen;
  for (int t = 0; t < n_threads; ++t) {
    job* j = &jobs[t];
    j->acc = acc; j->acc_bytes = acc_bytes; j->out_stage = out_stage; j->out_bytes = out_bytes;
    j->recv_stage = recv_stage; j->recv_bytes = recv_bytes; j->descs = descs; j->chosen = chosen;
    j->begin = n_chosen * (uint64_t)t / (uint64_t)n_threads;
    j->end = n_chosen * (uint64_t)(t + 1) / (uint64_t)n_threads;
    j->n_bits = n_bits; j->dtype = dtype; j->op = op; j->status = 0;
    if (pthread_create(&tid[t], NULL, worker, j) != 0) { status = ORC_E_ARG; break; }
    ++started;
  }
  for (int t = 0; t < started; ++t) {
    pthread_join(tid[t], NULL);
    if (jobs[t].status < 0 && status >= 0) status = jobs[t].status;
  }
  free(chosen);
  return status;
}
