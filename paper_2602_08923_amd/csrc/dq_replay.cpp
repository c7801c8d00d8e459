// Hop replay: the reduce-scatter schedules of Section 3.4 ("Reduce-scatter", "Fused
// kernels") and Appendix B run for N simulated workers whose gradients all sit in this
// GPU's HBM.  A transfer between workers is a pointer hand-off: the buffer one worker's
// kernel writes at step t is the packed_in of the receiving worker's kernel at step t+1.
// Every step is one launch (two where a node both forwards and keeps) whose grid covers
// all (worker, chunk) jobs of that step; the job tables are built once, here, on the host.
#include <string.h>

#include <new>
#include <vector>

#include "dq_device.h"

namespace {

struct HostJob {
  const uint8_t *in;
  const void *local;
  const float *mu;
  const uint32_t *src = nullptr;
  const uint32_t *dest = nullptr;
  const float *back = nullptr;
  void *out;
  uint64_t first_sg;
  uint32_t n_sg[4];
  uint32_t rank;
};

struct Launch {
  dq::Kind kind;
  dq_dtype dtype;  // dtype of `local`
  bool has_local = true;  // false: decompress without accumulation
  bool gather = false;    // some job reads its local super-groups through an index
  std::vector<HostJob> jobs;  // freed once the table is on the device
  uint32_t n_jobs = 0;
  size_t table_off = 0;  // byte offset of this launch's job table in scratch
  uint32_t max_tiles = 0;
  uint64_t total_tiles = 0;
  uint64_t max_entries = 0;
  uint64_t entries = 0;
};

struct Step {
  std::vector<Launch> launches;
};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Plan {
  std::vector<Step> steps;
  size_t scratch_bytes = 0;
  // ring and chain only: where the message of (bucket, chunk) sits inside a message set, its size, and
  // the two sets' starts (step t writes set t & 1); what dq_replay_message answers from
  std::vector<size_t> ring_slot, ring_bytes;
  uint8_t *ring_msg[2] = {nullptr, nullptr};
  uint32_t ring_chunks = 0;   // chunks per bucket (0: not a ring or chain)
  uint32_t ring_message_steps = 0;  // steps 0 .. this-1 write messages
};

bool is_mx(dq_codec c) { return c == DQ_MXFP8_E4M3 || c == DQ_MXFP6_E3M2 || c == DQ_MXFP4_E2M1; }

size_t chunk_bytes(dq_codec codec, const uint32_t n_sg[4]) {
  if (is_mx(codec)) return dq_mx_packed_bytes(codec, ((uint64_t)n_sg[0] + n_sg[1] + n_sg[2] + n_sg[3]) * 256);
  dq_chunk ch{0, {n_sg[0], n_sg[1], n_sg[2], n_sg[3]}};
  return dq_packed_bytes(&ch);
}

size_t elt_size(dq_dtype t) { return t == DQ_F32 ? 4 : 2; }

// Width counts of chunk c (of n equal chunks) of a reordered bucket: 2-bit SGs first,
// then 4-bit, 8-bit and 16-bit.
void chunk_widths(const uint32_t by_width[4], uint64_t m, uint32_t c, uint32_t out[4]) {
  uint64_t edges[5] = {0, 0, 0, 0, 0};
  for (int w = 0; w < 4; ++w) edges[w + 1] = edges[w] + by_width[w];
  const uint64_t lo = (uint64_t)c * m, hi = lo + m;
  for (int w = 0; w < 4; ++w) {
    const uint64_t a = lo > edges[w] ? lo : edges[w], b = hi < edges[w + 1] ? hi : edges[w + 1];
    out[w] = b > a ? (uint32_t)(b - a) : 0;
  }
}

// Builds the whole schedule.  With base == nullptr only sizes are computed (pointers are
// offsets from zero); grads may then be null.
dq_status build_plan(const dq_ctx *ctx, const dq_replay_desc *d, const void *const *grads, uint8_t *base, float *out,
                     Plan *plan) {
  if (!ctx || !d) return DQ_EINVAL;
  const uint32_t n = ctx->cfg.n_workers;
  const bool mx = is_mx(d->codec);
  if (!mx && d->codec != DQ_DYNAMIQ) return DQ_EINVAL;
  if (d->dtype != DQ_F32 && d->dtype != DQ_BF16) return DQ_EINVAL;
  if (n < 2 || d->n_buckets < 1 || d->n_sg_bucket < 1) return DQ_EINVAL;
  if (!mx && !d->n_sg_by_width) return DQ_EINVAL;
  if (mx && d->mu) return DQ_EINVAL;  // the MX codec has no normalization
  if (mx && d->origin) return DQ_EINVAL;
  if (d->inputs_in_original_order && (!d->origin || d->topology == DQ_CHAIN)) return DQ_EINVAL;
  if ((reinterpret_cast<uintptr_t>(d->mu) & 3u) || (reinterpret_cast<uintptr_t>(d->origin) & 3u)) return DQ_EALIGN;
  if (d->topology == DQ_CHAIN) {
    if (d->n_buckets != 1) return DQ_EINVAL;
  } else if (d->topology == DQ_RING || d->topology == DQ_BUTTERFLY) {
    if (d->n_sg_bucket % n) return DQ_EINVAL;
    if (d->topology == DQ_BUTTERFLY && (n & (n - 1))) return DQ_EINVAL;
  } else {
    return DQ_EINVAL;
  }
  if (d->n_sg_bucket >= (1ull << 31)) return DQ_EUNSUPPORTED;
  const size_t es = elt_size(d->dtype);
  const uint64_t bucket_entries = d->n_sg_bucket * 256;
  const uint32_t n_chunks = d->topology == DQ_CHAIN ? 1 : n;
  const uint64_t m = d->n_sg_bucket / n_chunks;  // SGs per chunk
  const uint64_t chunk_entries = m * 256;

  // per (bucket, chunk): widths, packed size
  struct ChunkInfo {
    uint32_t n_sg[4];
    uint64_t first_sg;
    size_t bytes;
  };
  std::vector<ChunkInfo> ci((size_t)d->n_buckets * n_chunks);
  for (uint32_t b = 0; b < d->n_buckets; ++b) {
    uint32_t bw[4] = {(uint32_t)d->n_sg_bucket, 0, 0, 0};
    if (!mx) {
      memcpy(bw, d->n_sg_by_width + 4 * (size_t)b, sizeof(bw));
      if ((uint64_t)bw[0] + bw[1] + bw[2] + bw[3] != d->n_sg_bucket) return DQ_EINVAL;
    }
    for (uint32_t c = 0; c < n_chunks; ++c) {
      ChunkInfo &x = ci[(size_t)b * n_chunks + c];
      chunk_widths(bw, m, c, x.n_sg);
      x.first_sg = d->first_sg + (uint64_t)b * d->n_sg_bucket + (uint64_t)c * m;
      x.bytes = chunk_bytes(d->codec, x.n_sg);
    }
  }
  auto grad_ptr = [&](uint32_t w, uint32_t b, uint32_t c) -> const void * {
    const uint8_t *g = grads ? (const uint8_t *)grads[w] : nullptr;
    return g + ((uint64_t)b * bucket_entries + (uint64_t)c * chunk_entries) * es;
  };
  auto out_ptr = [&](uint32_t b, uint32_t c) -> float * {
    return out + (uint64_t)b * bucket_entries + (uint64_t)c * chunk_entries;
  };
  // raw: `local` is a worker's own gradient (its means are still to be taken off), not an fp32
  // buffer of sums that already had them taken off
  auto mk = [&](const ChunkInfo &x, const uint8_t *in, const void *local, bool raw, void *o, uint32_t rank) {
    HostJob j;
    j.in = in;
    j.local = local;
    j.mu = (raw && d->mu) ? d->mu + (x.first_sg - d->first_sg) : nullptr;
    if (raw && d->inputs_in_original_order) {
      // `local` points at the chunk's place in a reordered bucket: step back to the bucket's start (the chunk
      // begins (first_sg - first of the bucket) super-groups in) and let the kernel gather through origin
      const uint64_t in_bucket = (x.first_sg - d->first_sg) % d->n_sg_bucket;
      j.local = static_cast<const uint8_t *>(local) - in_bucket * 256 * es;
      j.src = d->origin + (x.first_sg - d->first_sg);
    }
    j.out = o;
    j.first_sg = x.first_sg;
    memcpy(j.n_sg, x.n_sg, sizeof(j.n_sg));
    j.rank = rank;
    return j;
  };
  // The launch that writes the final result: with d->origin every super-group goes straight to its
  // original place in its bucket and gets its mean back (the restore, fused into the last kernel).
  auto finish = [&](HostJob j, const ChunkInfo &x, uint32_t b) {
    if (d->origin) {
      j.out = out + (uint64_t)b * bucket_entries;
      j.dest = d->origin + (x.first_sg - d->first_sg);
      j.back = d->mu ? d->mu + (x.first_sg - d->first_sg) : nullptr;
    }
    return j;
  };

  size_t off = 0;  // running scratch offset (job tables are appended at the end)
  plan->steps.clear();

  if (d->topology == DQ_CHAIN || d->topology == DQ_RING) {
    // two message sets (ping-pong), each with one slot per (bucket, chunk)
    std::vector<size_t> slot(ci.size());
    size_t set_bytes = 0;
    for (size_t i = 0; i < ci.size(); ++i) {
      slot[i] = set_bytes;
      set_bytes += align_up(ci[i].bytes, 256);
    }
    uint8_t *msg[2] = {base + off, base + off + set_bytes};
    off += 2 * set_bytes;
    plan->ring_slot = slot;
    plan->ring_bytes.resize(ci.size());
    for (size_t i = 0; i < ci.size(); ++i) plan->ring_bytes[i] = ci[i].bytes;
    plan->ring_msg[0] = msg[0];
    plan->ring_msg[1] = msg[1];
    plan->ring_chunks = n_chunks;
    plan->ring_message_steps = n - 1;
    const uint32_t hops = n;  // steps 0 .. n-1
    for (uint32_t t = 0; t < hops; ++t) {
      Step st;
      Launch L;
      L.dtype = d->dtype;
      L.kind = t == 0 ? dq::kCompress : (t == n - 1 ? dq::kDecompress : dq::kDar);
      for (uint32_t b = 0; b < d->n_buckets; ++b)
        for (uint32_t c = 0; c < n_chunks; ++c) {
          const size_t i = (size_t)b * n_chunks + c;
          // ring: chunk c is at worker c+t at step t; chain: slice t of the one chunk
          const uint32_t w = d->topology == DQ_CHAIN ? t : (c + t) % n;
          const void *local = d->topology == DQ_CHAIN ? grad_ptr(w, 0, 0) : grad_ptr(w, b, c);
          const uint8_t *in = t == 0 ? nullptr : msg[(t - 1) & 1] + slot[i];
          void *o = t == n - 1 ? (void *)out_ptr(b, c) : (void *)(msg[t & 1] + slot[i]);
          HostJob j = mk(ci[i], in, local, true, o, w);
          if (t == n - 1 && !d->all_gather) j = finish(j, ci[i], b);
          L.jobs.push_back(j);
        }
      st.launches.push_back(std::move(L));
      plan->steps.push_back(std::move(st));
    }
  } else {  // butterfly: recursive halving
    uint32_t Lg = 0;
    while ((1u << Lg) < n) ++Lg;
    // message region written at step k for receiver p: the chunks of p's keep range at step k
    // keep_lo(p, k): the chunks worker p still owns after step k
    auto keep_lo = [&](uint32_t p, uint32_t k) { return p & ~((n >> k) - 1); };
    // message sets: parity by step; region offsets per (bucket, receiver, chunk)
    std::vector<std::vector<size_t>> moff(Lg + 1);  // [k][(b*n + p)*half + (c - keep_lo)]
    size_t set_bytes[2] = {0, 0};
    for (uint32_t k = 1; k <= Lg; ++k) {
      const uint32_t half = n >> k;
      moff[k].resize((size_t)d->n_buckets * n * half);
      size_t o = 0;
      for (uint32_t b = 0; b < d->n_buckets; ++b)
        for (uint32_t p = 0; p < n; ++p)
          for (uint32_t j = 0; j < half; ++j) {
            moff[k][((size_t)b * n + p) * half + j] = o;
            o += align_up(ci[(size_t)b * n + keep_lo(p, k) + j].bytes, 256);
          }
      if (o > set_bytes[k & 1]) set_bytes[k & 1] = o;
    }
    uint8_t *msg[2] = {base + off, base + off + set_bytes[0]};
    off += set_bytes[0] + set_bytes[1];
    // fp32 keep-buffers: worker w, bucket b: the n/4 chunks it owns after step 2
    const uint32_t keep_chunks = n >= 4 ? n / 4 : 0;
    off = align_up(off, 256);
    float *acc = reinterpret_cast<float *>(base + off);
    off += (size_t)d->n_buckets * n * keep_chunks * chunk_entries * 4;
    auto acc_ptr = [&](uint32_t w, uint32_t b, uint32_t c) -> float * {
      return acc + (((uint64_t)b * n + w) * keep_chunks + (c - keep_lo(w, 2))) * chunk_entries;
    };
    auto msg_ptr = [&](uint32_t k, uint32_t b, uint32_t p, uint32_t c) -> uint8_t * {
      const uint32_t half = n >> k;
      return msg[k & 1] + moff[k][((size_t)b * n + p) * half + (c - keep_lo(p, k))];
    };
    for (uint32_t k = 1; k <= Lg; ++k) {
      const uint32_t half = n >> k;
      Step st;
      Launch send, keep;
      send.kind = k == 1 ? dq::kCompress : dq::kDar;
      keep.kind = dq::kDecompress;
      send.dtype = keep.dtype = (k <= 2) ? d->dtype : DQ_F32;  // later steps add into fp32 buffers
      for (uint32_t b = 0; b < d->n_buckets; ++b)
        for (uint32_t w = 0; w < n; ++w) {
          const uint32_t klo = keep_lo(w, k), partner = w ^ half;
          const uint32_t slo = klo ^ half;  // the other half of the range owned after step k-1
          for (uint32_t c = slo; c < slo + half; ++c) {
            const ChunkInfo &x = ci[(size_t)b * n + c];
            const uint8_t *in = k == 1 ? nullptr : msg_ptr(k - 1, b, w, c);
            const void *local = k <= 2 ? grad_ptr(w, b, c) : (const void *)acc_ptr(w, b, c);
            send.jobs.push_back(mk(x, in, local, k <= 2, msg_ptr(k, b, partner, c), w));
          }
          if (k >= 2)
            for (uint32_t c = klo; c < klo + half; ++c) {
              const ChunkInfo &x = ci[(size_t)b * n + c];
              const void *local = k == 2 ? grad_ptr(w, b, c) : (const void *)acc_ptr(w, b, c);
              keep.jobs.push_back(mk(x, msg_ptr(k - 1, b, w, c), local, k == 2, acc_ptr(w, b, c), w));
            }
        }
      st.launches.push_back(std::move(send));
      if (k >= 2) st.launches.push_back(std::move(keep));
      plan->steps.push_back(std::move(st));
    }
    // after the last exchange: worker w adds what it received for chunk w
    Step st;
    Launch fin;
    fin.kind = dq::kDecompress;
    fin.dtype = Lg == 1 ? d->dtype : DQ_F32;
    for (uint32_t b = 0; b < d->n_buckets; ++b)
      for (uint32_t w = 0; w < n; ++w) {
        const ChunkInfo &x = ci[(size_t)b * n + w];
        const void *local = Lg == 1 ? grad_ptr(w, b, w) : (const void *)acc_ptr(w, b, w);
        HostJob j = mk(x, msg_ptr(Lg, b, w, w), local, Lg == 1, out_ptr(b, w), w);
        if (!d->all_gather) j = finish(j, x, b);
        fin.jobs.push_back(j);
      }
    st.launches.push_back(std::move(fin));
    plan->steps.push_back(std::move(st));
  }

  if (d->all_gather) {
    // All-gather phase: the sink of each chunk compresses its fp32 sum (with its own rank: it has
    // compressed nothing of this chunk before, so these random numbers are fresh), and every
    // worker, the sink included, ends with the decompressed message.
    std::vector<size_t> slot(ci.size());
    off = align_up(off, 256);
    size_t region = 0;
    for (size_t i = 0; i < ci.size(); ++i) {
      slot[i] = region;
      region += align_up(ci[i].bytes, 256);
    }
    uint8_t *ag = base + off;
    off += region;
    Step sc, sd;
    Launch comp, dec;
    comp.kind = dq::kCompress;
    comp.dtype = DQ_F32;
    dec.kind = dq::kDecompress;
    dec.dtype = DQ_F32;
    dec.has_local = false;
    for (uint32_t b = 0; b < d->n_buckets; ++b)
      for (uint32_t c = 0; c < n_chunks; ++c) {
        const size_t i = (size_t)b * n_chunks + c;
        const uint32_t sink = d->topology == DQ_CHAIN ? n - 1 : (d->topology == DQ_RING ? (c + n - 1) % n : c);
        comp.jobs.push_back(mk(ci[i], nullptr, out_ptr(b, c), false, ag + slot[i], sink));
        dec.jobs.push_back(finish(mk(ci[i], ag + slot[i], nullptr, false, out_ptr(b, c), sink), ci[i], b));
      }
    sc.launches.push_back(std::move(comp));
    sd.launches.push_back(std::move(dec));
    plan->steps.push_back(std::move(sc));
    plan->steps.push_back(std::move(sd));
  }

  // job tables
  for (Step &st : plan->steps)
    for (Launch &L : st.launches) {
      off = align_up(off, 256);
      L.table_off = off;
      L.n_jobs = (uint32_t)L.jobs.size();
      off += L.jobs.size() * (mx ? sizeof(dq::MxJob) : sizeof(dq::Job));
      for (const HostJob &j : L.jobs) {
        if (j.src) L.gather = true;
        const uint32_t tiles = (j.n_sg[0] + 3) / 4 + (j.n_sg[1] + 3) / 4 + (j.n_sg[2] + 3) / 4 + (j.n_sg[3] + 3) / 4;
        const uint64_t e = ((uint64_t)j.n_sg[0] + j.n_sg[1] + j.n_sg[2] + j.n_sg[3]) * 256;
        if (tiles > L.max_tiles) L.max_tiles = tiles;
        L.total_tiles += tiles;
        if (e > L.max_entries) L.max_entries = e;
        L.entries += e;
      }
    }
  plan->scratch_bytes = align_up(off, 256);
  return DQ_OK;
}

}  // namespace

struct dq_replay {
  dq_ctx *ctx;
  dq_codec codec;
  Plan plan;
  uint8_t *scratch;
  std::vector<hipEvent_t> events;
};

extern "C" {

size_t dq_replay_scratch_bytes(const dq_ctx *ctx, const dq_replay_desc *desc) {
  Plan p;
  if (build_plan(ctx, desc, nullptr, nullptr, nullptr, &p) != DQ_OK) return 0;
  return p.scratch_bytes;
}

dq_status dq_replay_create(dq_ctx *ctx, const dq_replay_desc *desc, const void *const *worker_grads, void *scratch,
                           size_t scratch_bytes, float *out, dq_replay **plan_out) {
  if (!ctx || !desc || !worker_grads || !scratch || !out || !plan_out) return DQ_EINVAL;
  *plan_out = nullptr;
  if (desc->n_grads != 0 && desc->n_grads != ctx->cfg.n_workers) return DQ_EINVAL;
  if ((reinterpret_cast<uintptr_t>(scratch) & 255u) || (reinterpret_cast<uintptr_t>(out) & 15u)) return DQ_EALIGN;
  for (uint32_t w = 0; w < ctx->cfg.n_workers; ++w) {
    if (!worker_grads[w]) return DQ_EINVAL;
    if (reinterpret_cast<uintptr_t>(worker_grads[w]) & 15u) return DQ_EALIGN;
  }
  dq_replay *r = new (std::nothrow) dq_replay;
  if (!r) return DQ_EINVAL;
  r->ctx = ctx;
  r->codec = desc->codec;
  r->scratch = static_cast<uint8_t *>(scratch);
  dq_status st = build_plan(ctx, desc, worker_grads, r->scratch, out, &r->plan);
  if (st == DQ_OK && r->plan.scratch_bytes > scratch_bytes) st = DQ_EINVAL;
  if (st != DQ_OK) {
    delete r;
    return st;
  }
  const bool mx = desc->codec != DQ_DYNAMIQ;
  for (Step &s : r->plan.steps)
    for (Launch &L : s.launches) {
      if (L.jobs.empty()) continue;
      hipError_t e;
      if (mx) {
        std::vector<dq::MxJob> t(L.jobs.size());
        for (size_t i = 0; i < t.size(); ++i) {
          const HostJob &j = L.jobs[i];
          t[i] = dq::MxJob{j.in, j.local, j.out, ((uint64_t)j.n_sg[0] + j.n_sg[1] + j.n_sg[2] + j.n_sg[3]) * 256};
        }
        e = hipMemcpy(r->scratch + L.table_off, t.data(), t.size() * sizeof(dq::MxJob), hipMemcpyHostToDevice);
      } else {
        std::vector<dq::Job> t(L.jobs.size());
        for (size_t i = 0; i < t.size(); ++i) {
          const HostJob &j = L.jobs[i];
          t[i] = dq::make_job(j.in, j.local, j.mu, j.out, j.first_sg, j.n_sg, j.rank);
          t[i].src = j.src;
          t[i].dest = j.dest;
          t[i].back = j.back;
        }
        e = hipMemcpy(r->scratch + L.table_off, t.data(), t.size() * sizeof(dq::Job), hipMemcpyHostToDevice);
      }
      if (e != hipSuccess) {
        delete r;
        return dq::hip_status(e);
      }
      std::vector<HostJob>().swap(L.jobs);
    }
  *plan_out = r;
  return DQ_OK;
}

uint32_t dq_replay_n_steps(const dq_replay *plan) { return plan ? (uint32_t)plan->plan.steps.size() : 0; }

dq_status dq_replay_step_info(const dq_replay *plan, uint32_t step, uint32_t *kind, uint64_t *entries_dar,
                              uint64_t *entries_other) {
  if (!plan || step >= plan->plan.steps.size()) return DQ_EINVAL;
  uint64_t dar = 0, other = 0;
  uint32_t k = 0;
  bool has_dar = false, has_da = false, has_c = false;
  for (const Launch &L : plan->plan.steps[step].launches) {
    if (L.kind == dq::kDar) { dar += L.entries; has_dar = true; }
    else { other += L.entries; (L.kind == dq::kCompress ? has_c : has_da) = true; }
  }
  k = has_dar ? (has_da ? 3 : 1) : (has_c ? 0 : 2);
  if (kind) *kind = k;
  if (entries_dar) *entries_dar = dar;
  if (entries_other) *entries_other = other;
  return DQ_OK;
}

// only: -1 = every launch of the step, else the index of the one launch to enqueue
static dq_status run_step(dq_replay *plan, size_t i, hipStream_t s, int only = -1) {
  const bool mx = plan->codec != DQ_DYNAMIQ;
  int index = -1;
  for (const Launch &L : plan->plan.steps[i].launches) {
    ++index;
    if (only >= 0 && index != only) continue;
    if (L.n_jobs == 0) continue;
    hipError_t e;
    if (mx)
      e = dq::mx_launch_batch(L.kind, plan->codec, L.dtype, L.has_local,
                              reinterpret_cast<const dq::MxJob *>(plan->scratch + L.table_off),
                              L.n_jobs, L.max_entries, plan->ctx->n_cu, s);
    else
      e = dq::launch_batch(L.kind, L.dtype, L.has_local, L.gather, reinterpret_cast<const dq::Job *>(plan->scratch + L.table_off),
                           L.n_jobs, L.max_tiles, L.total_tiles, plan->ctx->params, plan->ctx->grid_blocks, s);
    if (e != hipSuccess) return dq::hip_status(e);
  }
  return DQ_OK;
}

dq_status dq_replay_run_steps(dq_replay *plan, uint32_t first, uint32_t count, void *hip_stream) {
  if (!plan || (size_t)first + count > plan->plan.steps.size()) return DQ_EINVAL;
  for (uint32_t i = first; i < first + count; ++i) {
    const dq_status st = run_step(plan, i, (hipStream_t)hip_stream);
    if (st != DQ_OK) return st;
  }
  return DQ_OK;
}

dq_status dq_replay_run_launch(dq_replay *plan, uint32_t step, uint32_t launch, void *hip_stream) {
  if (!plan || step >= plan->plan.steps.size() || launch >= plan->plan.steps[step].launches.size()) return DQ_EINVAL;
  return run_step(plan, step, (hipStream_t)hip_stream, (int)launch);
}

dq_status dq_replay_run(dq_replay *plan, float *step_ms, void *hip_stream) {
  if (!plan) return DQ_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  const size_t ns = plan->plan.steps.size();
  hipError_t he = hipSuccess;
  while (step_ms && he == hipSuccess && plan->events.size() < ns + 1) {
    hipEvent_t e;
    he = hipEventCreate(&e);
    if (he == hipSuccess) plan->events.push_back(e);
  }
  if (step_ms && he == hipSuccess) he = hipEventRecord(plan->events[0], s);
  for (size_t i = 0; i < ns && he == hipSuccess; ++i) {
    const dq_status st = run_step(plan, i, s);
    if (st != DQ_OK) return st;
    if (step_ms) he = hipEventRecord(plan->events[i + 1], s);
  }
  if (step_ms && he == hipSuccess) he = hipEventSynchronize(plan->events[ns]);
  for (size_t i = 0; step_ms && i < ns && he == hipSuccess; ++i)
    he = hipEventElapsedTime(&step_ms[i], plan->events[i], plan->events[i + 1]);
  return dq::hip_status(he);
}

dq_status dq_replay_message(const dq_replay *plan, uint32_t step, uint32_t bucket, uint32_t chunk, const void **ptr,
                            size_t *bytes) {
  if (!plan || !ptr || !bytes) return DQ_EINVAL;
  const Plan &p = plan->plan;
  if (p.ring_chunks == 0) return DQ_EUNSUPPORTED;
  const size_t i = (size_t)bucket * p.ring_chunks + chunk;
  if (step >= p.ring_message_steps || chunk >= p.ring_chunks || i >= p.ring_slot.size()) return DQ_EINVAL;
  *ptr = p.ring_msg[step & 1] + p.ring_slot[i];
  *bytes = p.ring_bytes[i];
  return DQ_OK;
}

void dq_replay_destroy(dq_replay *plan) {
  if (!plan) return;
  for (hipEvent_t e : plan->events) (void)hipEventDestroy(e);
  delete plan;
}

}  // extern "C"
