// Double-buffered pass over a long gradient (Sec. 5, "Protocol": quantization and
// communication of one part overlap with work on the next).  The vector is cut into
// chunks that are multiples of the bucket size; the K encodes of chunk j+1 run on one
// stream while decode + step of chunk j runs on another, with two sets of message
// buffers used alternately.  Buckets and draw indices are those of the whole vector,
// so x ends up bit for bit as after one flat qsgd_sgd_step.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <new>

#include "qsgd.h"
#include "qsgd_kernels.hpp"

struct qsgd_pipeline {
  hipStream_t enc = nullptr, dec = nullptr;
  hipEvent_t start = nullptr;        // the caller's stream at the time of the call
  hipEvent_t encoded[2] = {nullptr, nullptr};
  hipEvent_t decoded[2] = {nullptr, nullptr};
  int device = 0;
};

extern "C" {

int qsgd_pipeline_create(qsgd_pipeline** out) {
  if (!out) return QSGD_ERR_INVALID_ARG;
  qsgd_pipeline* pl = new (std::nothrow) qsgd_pipeline;
  if (!pl) return QSGD_ERR_INVALID_ARG;
  bool ok = hipGetDevice(&pl->device) == hipSuccess &&
            hipStreamCreateWithFlags(&pl->enc, hipStreamNonBlocking) == hipSuccess &&
            hipStreamCreateWithFlags(&pl->dec, hipStreamNonBlocking) == hipSuccess &&
            hipEventCreateWithFlags(&pl->start, hipEventDisableTiming) == hipSuccess;
  for (int i = 0; ok && i < 2; ++i)
    ok = hipEventCreateWithFlags(&pl->encoded[i], hipEventDisableTiming) == hipSuccess &&
         hipEventCreateWithFlags(&pl->decoded[i], hipEventDisableTiming) == hipSuccess;
  if (!ok) { qsgd_pipeline_destroy(pl); return QSGD_ERR_HIP; }
  *out = pl;
  return QSGD_OK;
}

void qsgd_pipeline_destroy(qsgd_pipeline* pl) {
  if (!pl) return;
  if (pl->enc) { (void)hipStreamSynchronize(pl->enc); (void)hipStreamDestroy(pl->enc); }
  if (pl->dec) { (void)hipStreamSynchronize(pl->dec); (void)hipStreamDestroy(pl->dec); }
  if (pl->start) (void)hipEventDestroy(pl->start);
  for (int i = 0; i < 2; ++i) {
    if (pl->encoded[i]) (void)hipEventDestroy(pl->encoded[i]);
    if (pl->decoded[i]) (void)hipEventDestroy(pl->decoded[i]);
  }
  delete pl;
}

int qsgd_pipeline_step(qsgd_pipeline* pl, const qsgd_params* p, uint64_t chunk_elems,
                       const float* const* g_dev, uint32_t K, float eta, float* x_dev,
                       void* const* msg_dev, size_t msg_capacity, void* enc_workspace_dev,
                       void* dec_workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!pl || !p || !g_dev || !msg_dev || K < 1 || K > QSGD_MAX_PEERS || !x_dev ||
      !enc_workspace_dev || !dec_workspace_dev || enc_workspace_dev == dec_workspace_dev)
    return QSGD_ERR_INVALID_ARG;
  const uint64_t d = p->n == 0 ? p->d : std::min<uint64_t>(p->d, p->n);
  // chunks are whole buckets, and every slice starts on a 16-byte boundary
  if (d < 1 || chunk_elems == 0 || chunk_elems % d || chunk_elems % 4) return QSGD_ERR_INVALID_ARG;
  // Every chunk is checked before anything is queued, so that an error leaves x untouched:
  // the full chunks share one geometry, the last one may be shorter.
  if (p->n > 0) {
    const uint64_t nchunks = (p->n + chunk_elems - 1) / chunk_elems;
    const uint64_t which[2] = {0, nchunks - 1};
    for (int i = 0; i < (nchunks > 1 ? 2 : 1); ++i) {
      const uint64_t off = which[i] * chunk_elems;
      qsgd_params pc = *p;
      pc.n = std::min<uint64_t>(chunk_elems, p->n - off);
      int rc = qsgd::validate_encode(&pc, off, msg_capacity, workspace_bytes);
      if (!rc) rc = qsgd::validate_decode(&pc, K, workspace_bytes);
      if (rc) return rc;
    }
  }
  auto aligned16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
  if (!aligned16(x_dev) || !aligned16(enc_workspace_dev) || !aligned16(dec_workspace_dev))
    return QSGD_ERR_INVALID_ARG;
  for (uint32_t k = 0; k < 2 * K; ++k)
    if (!msg_dev[k] || !aligned16(msg_dev[k])) return QSGD_ERR_INVALID_ARG;
  for (uint32_t k = 0; k < K; ++k)
    if (!g_dev[k] || !aligned16(g_dev[k])) return QSGD_ERR_INVALID_ARG;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return QSGD_ERR_HIP;
  if (dev != pl->device) return QSGD_ERR_INVALID_ARG;
  hipStream_t user = reinterpret_cast<hipStream_t>(hip_stream);
  // both streams start after what the caller has queued so far
  if (hipEventRecord(pl->start, user) != hipSuccess ||
      hipStreamWaitEvent(pl->enc, pl->start, 0) != hipSuccess ||
      hipStreamWaitEvent(pl->dec, pl->start, 0) != hipSuccess)
    return QSGD_ERR_HIP;

  const float c_eta = eta;   // every chunk applies eta / K to its own slice
  size_t sizes[QSGD_MAX_PEERS];
  const void* set[QSGD_MAX_PEERS];
  for (uint32_t k = 0; k < K; ++k) sizes[k] = msg_capacity;
  uint64_t chunk = 0;
  for (uint64_t off = 0; off < p->n; off += chunk_elems, ++chunk) {
    const int sb = (int)(chunk & 1);
    qsgd_params pc = *p;
    pc.n = std::min<uint64_t>(chunk_elems, p->n - off);
    // message set sb is free again once chunk - 2 has been decoded
    if (chunk >= 2 && hipStreamWaitEvent(pl->enc, pl->decoded[sb], 0) != hipSuccess)
      return QSGD_ERR_HIP;
    for (uint32_t k = 0; k < K; ++k) {
      pc.stream_id = p->stream_id + k;
      const int rc = qsgd_encode_slice(&pc, off, g_dev[k] + off, msg_dev[sb * K + k], msg_capacity,
                                       enc_workspace_dev, workspace_bytes, pl->enc);
      if (rc) return rc;
      set[k] = msg_dev[sb * K + k];
    }
    if (hipEventRecord(pl->encoded[sb], pl->enc) != hipSuccess ||
        hipStreamWaitEvent(pl->dec, pl->encoded[sb], 0) != hipSuccess)
      return QSGD_ERR_HIP;
    pc.stream_id = p->stream_id;
    const int rc = qsgd_sgd_step(&pc, set, sizes, K, c_eta, x_dev + off, dec_workspace_dev,
                                 workspace_bytes, pl->dec);
    if (rc) return rc;
    if (hipEventRecord(pl->decoded[sb], pl->dec) != hipSuccess) return QSGD_ERR_HIP;
  }
  // the caller's stream continues after the last chunk
  if (chunk > 0) {
    const int last = (int)((chunk - 1) & 1);
    if (hipStreamWaitEvent(user, pl->decoded[last], 0) != hipSuccess) return QSGD_ERR_HIP;
    if (chunk > 1 && hipStreamWaitEvent(user, pl->decoded[last ^ 1], 0) != hipSuccess)
      return QSGD_ERR_HIP;
  }
  return QSGD_OK;
}

}  // extern "C"
