// Token routing and selection arrays (sections 2.1, 3.1, 4.1 "SEL", 6.2 shared experts).
//
// Four small kernels on the caller's stream (one fused kernel for up to 256 tokens):
//   route      one wavefront per token: softmax over E logits, top-k by repeated
//              wave arg-max on the logits (ties to the lower expert id)
//   histogram  one block per chunk of 256 tokens: tokens per expert in the chunk
//   scan       one block: expert offsets and the start of every (chunk, expert) run in its bucket
//   scatter    one block per chunk: stable position of every (token, slot) pair from
//              per-wavefront bit masks + population counts, then sel / sel_w / inv
// The bucket order (ascending token id inside an expert) is a stable counting sort,
// so the integer outputs are reproducible bit for bit.
#include "ssmm_common.h"

namespace ssmm {

constexpr int kChunk = 256;      // tokens per block in histogram / scatter
constexpr int kMaxExperts = 256;  // routed + shared
constexpr int kMaxTopk = 16;

__device__ inline float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ inline float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Routing of token t by one wavefront.  Lane l owns experts l, l+64, l+128, l+192; lane j < topk
// returns the j-th choice (expert id, weight).  A NaN logit counts as -infinity (a masked expert):
// weight 0, chosen only when fewer than topk logits are above -infinity, then by ascending id
// like any other tie; the ids of a token are always distinct.
__device__ inline float logit_or_minus_inf(float v) { return v != v ? -__builtin_huge_valf() : v; }
__device__ inline void route_token(const float* __restrict__ logits, int t, int E, int topk, int renormalize, int lane,
                                   int& out_id, float& out_w) {
  const float NEG = -__builtin_huge_valf();
  if (E <= 64) {
    // One expert per lane: a lane's place in the descending order (ties: lower id first) is the
    // number of experts that beat it, counted against every lane's logit in turn (64 broadcasts,
    // no dependent cross-lane chain).
    const float lg = lane < E ? logit_or_minus_inf(logits[(int64_t)t * E + lane]) : NEG;
    int place = 0;
    float mx = NEG;
#pragma unroll
    for (int o = 0; o < 64; o++) {
      const float v = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, lg), o));
      place += (v > lg || (v == lg && o < lane)) ? 1 : 0;
      mx = fmaxf(mx, v);
    }
    if (lane >= E) place = 64;   // padding lanes never rank (their -inf would tie with a real -inf logit)
    const float pr = lane < E ? expf(lg - mx) : 0.f;
    const float inv_sum = 1.0f / wave_sum(pr);
    const float w = pr * inv_sum;
    const float chosen_sum = wave_sum(place < topk ? w : 0.f);
    // lane j takes the lane whose place is j (its number is the expert id) and that lane's weight
    int my_id = 0;
    float my_w = 0.f;
    for (int j = 0; j < topk; j++) {
      const int src = __builtin_ctzll(__ballot(place == j));
      const float wj = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w), src));
      if (lane == j) {
        my_id = src;
        my_w = wj;
      }
    }
    out_id = my_id;
    out_w = renormalize ? my_w / chosen_sum : my_w;
    return;
  }
  float lg[4], pr[4];
  for (int i = 0; i < 4; i++) {
    const int e = lane + 64 * i;
    lg[i] = e < E ? logit_or_minus_inf(logits[(int64_t)t * E + e]) : NEG;
  }
  const float mx = wave_max(fmaxf(fmaxf(lg[0], lg[1]), fmaxf(lg[2], lg[3])));
  float s = 0.f;
  for (int i = 0; i < 4; i++) {
    pr[i] = lane + 64 * i < E ? expf(lg[i] - mx) : 0.f;
    s += pr[i];
  }
  const float inv_sum = 1.0f / wave_sum(s);
  float my_w = 0.f;   // lane j keeps the j-th choice
  int my_id = 0;
  float chosen_sum = 0.f;
  // bit i of `open`: expert lane + 64 i exists and has not been chosen yet (a chosen expert is
  // struck out here, not by overwriting its logit: -infinity is a legal logit that may still be
  // chosen, once, when fewer than topk experts are above it)
  uint32_t open = 0;
  for (int i = 0; i < 4; i++)
    if (lane + 64 * i < E) open |= 1u << i;
  const int kNone = 1 << 30;   // id of "no candidate": loses every tie
  for (int j = 0; j < topk; j++) {
    // lane-local best among the open experts (lower expert id first on equal logits), then across the wave
    float bv = NEG;
    int bi = kNone;
    float bp = 0.f;
    for (int i = 0; i < 4; i++)
      if (((open >> i) & 1u) && (bi == kNone || lg[i] > bv)) {
        bv = lg[i];
        bi = lane + 64 * i;
        bp = pr[i];
      }
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(bv, o, 64);
      const int oi = __shfl_xor(bi, o, 64);
      const float op = __shfl_xor(bp, o, 64);
      if (ov > bv || (ov == bv && oi < bi)) {
        bv = ov;
        bi = oi;
        bp = op;
      }
    }
    const float w = bp * inv_sum;
    chosen_sum += w;
    if (lane == j) {
      my_w = w;
      my_id = bi;
    }
    for (int i = 0; i < 4; i++)
      if (bi == lane + 64 * i) open &= ~(1u << i);   // strike the winner out
  }
  out_id = my_id;
  out_w = renormalize ? my_w / chosen_sum : my_w;
}

// One wavefront per token.
__global__ void __launch_bounds__(256) route_kernel(const float* __restrict__ logits, int T, int E, int topk,
                                                    int renormalize, int32_t* __restrict__ topk_ids,
                                                    float* __restrict__ topk_w) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  int id;
  float w;
  route_token(logits, t, E, topk, renormalize, lane, id, w);
  if (lane < topk) {
    topk_ids[(int64_t)t * topk + lane] = id;
    topk_w[(int64_t)t * topk + lane] = w;
  }
}

// counts[c][e] = tokens of chunk c routed to expert e.
__global__ void __launch_bounds__(kChunk) histogram_kernel(const int32_t* __restrict__ topk_ids, int T, int E,
                                                           int topk, int32_t* __restrict__ counts) {
  __shared__ int hist[kMaxExperts];
  for (int e = threadIdx.x; e < E; e += kChunk) hist[e] = 0;
  __syncthreads();
  const int t = blockIdx.x * kChunk + threadIdx.x;
  if (t < T)
    for (int j = 0; j < topk; j++) atomicAdd(&hist[topk_ids[(int64_t)t * topk + j]], 1);
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += kChunk) counts[(int64_t)blockIdx.x * E + e] = hist[e];
}

// One block of 16 wavefronts.  Wavefront w takes experts w, w+16, ...: lane c holds the count of
// chunk c (64 chunks per round, a carry between rounds) and a wavefront scan turns the counts into
// the start of every (chunk, expert) run inside the expert's bucket; wavefront 0 then scans the
// expert totals (four experts per lane) into expert_offsets.
__device__ inline int wave_inclusive_scan(int v, int lane) {
  for (int o = 1; o < 64; o <<= 1) {
    const int u = __shfl_up(v, o, 64);
    if (lane >= o) v += u;
  }
  return v;
}
__global__ void __launch_bounds__(1024) scan_kernel(int32_t* __restrict__ counts /* in: counts, out: run starts in the bucket */,
                                                    int chunks, int T, int E, int n_shared,
                                                    int32_t* __restrict__ expert_offsets) {
  __shared__ int total[kMaxExperts];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int e = wave; e < E; e += 16) {
    int carry = 0;
    for (int c0 = 0; c0 < chunks; c0 += 64) {
      const int c = c0 + lane;
      const int n = c < chunks ? counts[(int64_t)c * E + e] : 0;
      const int incl = wave_inclusive_scan(n, lane);
      if (c < chunks) counts[(int64_t)c * E + e] = carry + incl - n;
      carry += __builtin_amdgcn_readlane(incl, 63);
    }
    if (lane == 0) total[e] = carry;
  }
  __syncthreads();
  if (wave == 0) {
    int v[4], sum = 0;
    for (int i = 0; i < 4; i++) {
      v[i] = lane * 4 + i < E ? total[lane * 4 + i] : 0;
      sum += v[i];
    }
    const int incl = wave_inclusive_scan(sum, lane);
    int s = incl - sum;
    for (int i = 0; i < 4; i++) {
      if (lane * 4 + i < E) expert_offsets[lane * 4 + i] = s;
      s += v[i];
    }
    const int routed = __builtin_amdgcn_readlane(incl, 63);
    for (int i = lane; i <= n_shared; i += 64) expert_offsets[E + i] = routed + i * T;   // shared expert i holds all T tokens
  }
}

// Position of a (token, expert) pair inside its chunk's run: the number of lower tokens of the
// chunk that chose the expert.  Every wavefront keeps one 64-bit mask per expert (bit l: the token of
// lane l chose it; set with LDS atomic ORs, whose result does not depend on their order), so the
// position is a population count below the lane plus the counts of the wavefronts below.
__device__ inline void mark_choices(unsigned long long (*mask)[kMaxExperts], int wave, int lane, const int* ids, int topk) {
#pragma unroll
  for (int j = 0; j < kMaxTopk; j++)
    if (j < topk && ids[j] >= 0) atomicOr(&mask[wave][ids[j]], 1ull << lane);
}
__device__ inline int place_in_chunk(unsigned long long (*mask)[kMaxExperts], int wave, int lane, int e) {
  const unsigned long long below = lane == 0 ? 0 : (~0ull >> (64 - lane));
  int r = __popcll(mask[wave][e] & below);
  for (int w = 0; w < wave; w++) r += __popcll(mask[w][e]);
  return r;
}

__global__ void __launch_bounds__(kChunk) scatter_kernel(const int32_t* __restrict__ topk_ids,
                                                         const float* __restrict__ topk_w,
                                                         const int32_t* __restrict__ run_start,
                                                         const int32_t* __restrict__ expert_offsets, int T, int E,
                                                         int topk, int n_shared, int32_t* __restrict__ sel,
                                                         float* __restrict__ sel_w, int32_t* __restrict__ inv) {
  __shared__ unsigned long long mask[kChunk / 64][kMaxExperts];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x * kChunk + threadIdx.x;
  for (int i = threadIdx.x; i < (kChunk / 64) * E; i += kChunk) mask[i / E][i % E] = 0;
  int ids[kMaxTopk];
#pragma unroll
  for (int j = 0; j < kMaxTopk; j++) ids[j] = (t < T && j < topk) ? topk_ids[(int64_t)t * topk + j] : -1;
  __syncthreads();
  mark_choices(mask, wave, lane, ids, topk);
  __syncthreads();
  if (t >= T) return;
  const int slots = topk + n_shared;
#pragma unroll
  for (int j = 0; j < kMaxTopk; j++)
    if (j < topk) {
      const int e = ids[j];
      const int pos = expert_offsets[e] + run_start[(int64_t)blockIdx.x * E + e] + place_in_chunk(mask, wave, lane, e);
      sel[pos] = t;
      sel_w[pos] = topk_w[(int64_t)t * topk + j];
      inv[(int64_t)t * slots + j] = pos;
    }
  for (int s = 0; s < n_shared; s++) {
    const int pos = T * topk + s * T + t;
    sel[pos] = t;
    sel_w[pos] = 1.0f;
    inv[(int64_t)t * slots + topk + s] = pos;
  }
}

// Up to 256 tokens: one block of 16 wavefronts instead of three or four launches that cost more
// than the work.  Phase 1 (up to 64 tokens; beyond that route_kernel has run): wavefront w routes
// tokens w, w+16, ...; phase 2: thread t < 256 places token t exactly as histogram + scan + scatter
// do for a single chunk.
constexpr int kSmallT = kChunk;
__global__ void __launch_bounds__(1024) route_bucket_small_kernel(const float* __restrict__ logits, int T, int E, int topk,
                                                                  int n_shared, int renormalize, int do_route,
                                                                  int32_t* __restrict__ topk_ids, float* __restrict__ topk_w,
                                                                  int32_t* __restrict__ expert_offsets,
                                                                  int32_t* __restrict__ sel, float* __restrict__ sel_w,
                                                                  int32_t* __restrict__ inv) {
  __shared__ int ids_s[kSmallT][kMaxTopk];
  __shared__ float w_s[kSmallT][kMaxTopk];
  __shared__ unsigned long long mask[kChunk / 64][kMaxExperts];
  __shared__ int start[kMaxExperts + 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < (kChunk / 64) * E; i += 1024) mask[i / E][i % E] = 0;
  if (do_route) {
    for (int t = wave; t < T; t += 16) {
      int id;
      float w;
      route_token(logits, t, E, topk, renormalize, lane, id, w);
      if (lane < topk) {
        topk_ids[(int64_t)t * topk + lane] = id;
        topk_w[(int64_t)t * topk + lane] = w;
        ids_s[t][lane] = id;
        w_s[t][lane] = w;
      }
    }
  } else {   // routed by route_kernel (a wavefront per token in parallel: each token costs a memory round trip)
    for (int i = threadIdx.x; i < T * topk; i += 1024) {
      ids_s[i / topk][i % topk] = topk_ids[i];
      w_s[i / topk][i % topk] = topk_w[i];
    }
  }
  __syncthreads();
  const int t = threadIdx.x;
  int ids[kMaxTopk];
  if (t < kChunk) {   // wavefronts 0..3, whole
#pragma unroll
    for (int j = 0; j < kMaxTopk; j++) ids[j] = (t < T && j < topk) ? ids_s[t][j] : -1;
    mark_choices(mask, wave, lane, ids, topk);
  }
  __syncthreads();
  if (wave == 0) {   // bucket sizes, four experts per lane, scanned into the offsets
    int v[4], sum = 0;
    for (int i = 0; i < 4; i++) {
      const int e = lane * 4 + i;
      v[i] = 0;
      if (e < E)
        for (int w = 0; w < kChunk / 64; w++) v[i] += __popcll(mask[w][e]);
      sum += v[i];
    }
    const int incl = wave_inclusive_scan(sum, lane);
    int s = incl - sum;
    for (int i = 0; i < 4; i++) {
      if (lane * 4 + i < E) start[lane * 4 + i] = s;
      s += v[i];
    }
    if (lane == 63) start[E] = incl;
  }
  __syncthreads();
  if (t < E) expert_offsets[t] = start[t];
  if (t <= n_shared) expert_offsets[E + t] = start[E] + t * T;
  if (t >= T) return;
  const int slots = topk + n_shared;
#pragma unroll
  for (int j = 0; j < kMaxTopk; j++)
    if (j < topk) {
      const int e = ids[j];
      const int pos = start[e] + place_in_chunk(mask, wave, lane, e);
      sel[pos] = t;
      sel_w[pos] = w_s[t][j];
      inv[(int64_t)t * slots + j] = pos;
    }
  for (int sh = 0; sh < n_shared; sh++) {
    const int pos = T * topk + sh * T + t;
    sel[pos] = t;
    sel_w[pos] = 1.0f;
    inv[(int64_t)t * slots + topk + sh] = pos;
  }
}

__global__ void zero_offsets_kernel(int32_t* expert_offsets, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) expert_offsets[i] = 0;
}

}  // namespace ssmm

using namespace ssmm;

extern "C" size_t ssmm_route_workspace_bytes(int T, int E, int topk, int n_shared) {
  (void)topk;
  (void)n_shared;
  if (T < 0 || E < 1) return 0;
  const size_t chunks = ((size_t)T + kChunk - 1) / kChunk;
  return ((chunks * (size_t)E * sizeof(int32_t)) + 255) / 256 * 256 + 256;
}

namespace ssmm {

// Everything ssmm_route_bucket does, with the per-chunk histogram in `counts`
// (chunks x E cells; unused up to kSmallT tokens).  Arguments already checked.
static int launch_route_bucket(const float* logits, int T, int E, int topk, int n_shared, int renormalize,
                               int32_t* topk_ids, float* topk_w, int32_t* expert_offsets, int32_t* sel, float* sel_w,
                               int32_t* inv, int32_t* counts, hipStream_t s) {
  if (T <= kSmallT) {
    const int fused_route = T <= 16;   // one token per wavefront (measured: with more, routing them one after the other costs more than a launch)
    if (!fused_route) {
      hipLaunchKernelGGL(route_kernel, dim3((T + 3) / 4), dim3(256), 0, s, logits, T, E, topk, renormalize, topk_ids,
                         topk_w);
      SSMM_RETURN_IF_LAUNCH_FAILED();
    }
    hipLaunchKernelGGL(route_bucket_small_kernel, dim3(1), dim3(1024), 0, s, logits, T, E, topk, n_shared, renormalize,
                       fused_route, topk_ids, topk_w, expert_offsets, sel, sel_w, inv);
    SSMM_RETURN_IF_LAUNCH_FAILED();
    return SSMM_OK;
  }
  const int chunks = (T + kChunk - 1) / kChunk;
  hipLaunchKernelGGL(route_kernel, dim3((T + 3) / 4), dim3(256), 0, s, logits, T, E, topk, renormalize, topk_ids,
                     topk_w);
  SSMM_RETURN_IF_LAUNCH_FAILED();
  hipLaunchKernelGGL(histogram_kernel, dim3(chunks), dim3(kChunk), 0, s, (const int32_t*)topk_ids, T, E, topk,
                     counts);
  SSMM_RETURN_IF_LAUNCH_FAILED();
  hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, s, counts, chunks, T, E, n_shared, expert_offsets);
  SSMM_RETURN_IF_LAUNCH_FAILED();
  hipLaunchKernelGGL(scatter_kernel, dim3(chunks), dim3(kChunk), 0, s, (const int32_t*)topk_ids,
                     (const float*)topk_w, (const int32_t*)counts, (const int32_t*)expert_offsets, T, E, topk, n_shared, sel,
                     sel_w, inv);
  SSMM_RETURN_IF_LAUNCH_FAILED();
  return SSMM_OK;
}

// Host-side checks shared by the two entry points; SSMM_OK with *done set when nothing is left to do.
static int check_route_bucket(const float* logits, int T, int E, int topk, int n_shared, int32_t* topk_ids, float* topk_w,
                              int32_t* expert_offsets, int32_t* sel, float* sel_w, int32_t* inv, hipStream_t s, bool* done) {
  *done = false;
  if (T < 0 || E < 1 || n_shared < 0) return SSMM_EINVAL;
  if (topk < 1 || topk > E || topk > kMaxTopk) return SSMM_ESHAPE;
  if (E + n_shared > kMaxExperts) return SSMM_ESHAPE;
  if ((int64_t)T * (topk + n_shared) > INT32_MAX) return SSMM_ESHAPE;
  if (!expert_offsets) return SSMM_EINVAL;
  if (T == 0) {
    hipLaunchKernelGGL(zero_offsets_kernel, dim3(2), dim3(256), 0, s, expert_offsets, E + n_shared + 1);
    SSMM_RETURN_IF_LAUNCH_FAILED();
    *done = true;
    return SSMM_OK;
  }
  if (!logits || !topk_ids || !topk_w || !sel || !sel_w || !inv) return SSMM_EINVAL;
  return SSMM_OK;
}

// ---- the entry point that allocates nothing and takes no workspace -------------------------
// Its per-chunk histogram lives in this array, one copy per GPU, held until the process ends.
constexpr int kStaticCells = 65536;   // (chunks of 256 tokens) x E cells of 4 bytes: 256 KiB
static __device__ __align__(256) int32_t scratch[kStaticCells];

// In host code `scratch` is a stand-in, not a device address.  The device address is asked for
// once per device, with that device current, and kept; only that pointer goes to kernels.
constexpr int kMaxDevices = 64;
static int32_t* scratch_ptr[kMaxDevices];
static int scratch_of_current_device(int32_t** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SSMM_EHIP;
  int32_t* p = __atomic_load_n(&scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    void* addr = nullptr;
    if (hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)) != hipSuccess || !addr) return SSMM_EHIP;
    p = (int32_t*)addr;   // every thread that gets here is given the same address for this device
    __atomic_store_n(&scratch_ptr[dev], p, __ATOMIC_RELEASE);
  }
  *out = p;
  return SSMM_OK;
}

}  // namespace ssmm

extern "C" int ssmm_route_bucket(const float* logits, int T, int E, int topk, int n_shared, int renormalize,
                                 int32_t* topk_ids, float* topk_w, int32_t* expert_offsets, int32_t* sel,
                                 float* sel_w, int32_t* inv, void* workspace, size_t workspace_bytes,
                                 void* stream) {
  hipStream_t s = (hipStream_t)stream;
  bool done = false;
  const int st = check_route_bucket(logits, T, E, topk, n_shared, topk_ids, topk_w, expert_offsets, sel, sel_w, inv, s, &done);
  if (st || done) return st;
  if (!workspace) return SSMM_EINVAL;
  if (workspace_bytes < ssmm_route_workspace_bytes(T, E, topk, n_shared)) return SSMM_EWORKSPACE;
  return launch_route_bucket(logits, T, E, topk, n_shared, renormalize, topk_ids, topk_w, expert_offsets, sel, sel_w, inv,
                             (int32_t*)workspace, s);
}

extern "C" int ssmm_route_bucket_noalloc(const float* logits, int T, int E, int topk, int n_shared, int renormalize,
                                         int32_t* topk_ids, float* topk_w, int32_t* expert_offsets, int32_t* sel,
                                         float* sel_w, int32_t* inv, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  // the size limit first: it holds whatever else is wrong with the call
  if (T > 0 && E > 0 && ((int64_t)T + kChunk - 1) / kChunk * E > kStaticCells) return SSMM_ELIMIT;
  bool done = false;
  int st = check_route_bucket(logits, T, E, topk, n_shared, topk_ids, topk_w, expert_offsets, sel, sel_w, inv, s, &done);
  if (st || done) return st;
  int32_t* counts = nullptr;
  st = scratch_of_current_device(&counts);
  if (st) return st;
  // nothing in the array has to start at zero: histogram_kernel writes every cell scan_kernel reads
  return launch_route_bucket(logits, T, E, topk, n_shared, renormalize, topk_ids, topk_w, expert_offsets, sel, sel_w, inv,
                             counts, s);
}

// ---------------------------------------------------------------------------------------------
// Router (section 2.1: the gate network in front of the experts): logits[t][e] = sum over k of
// x[t][k] * Wr[e][k], bf16 operands, fp32 accumulation in a fixed order (repeatable bits: the
// top-k decision hangs on them).  One block per 32 tokens and all experts (tiles of 32), its
// wavefronts split the reduction and their partial sums are added in wavefront order; dense MFMA
// 32x32x16: lane (i, q) = (lane % 32, lane / 32) feeds row i with reduction elements
// 8q..8q+7 of each 16-element step, for both operands; accumulator register r of lane (j, q)
// is output row (r % 4) + 4 q + 8 (r / 4), column j.
// ---------------------------------------------------------------------------------------------
namespace ssmm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 rt_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float rt_f32x16;

constexpr int kRouterWaves = 8;   // wavefronts of a block: each takes a slice of the reduction

template <int NE>   // expert tiles of 32
__global__ void __launch_bounds__(64 * kRouterWaves) router_logits_kernel(const uint16_t* __restrict__ x, int T, int H,
                                                                          const uint16_t* __restrict__ wr, int E,
                                                                          float* __restrict__ logits) {
  __shared__ float part[kRouterWaves][1024];   // one 32 x 32 tile of partial sums per wavefront
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t0 = blockIdx.x * 32;
  const int i = lane & 31, q = lane >> 5;
  const int steps = H / 16, k0 = 16 * (wave * steps / kRouterWaves), k1 = 16 * ((wave + 1) * steps / kRouterWaves);
  const uint16_t* xrow = x + (int64_t)min(t0 + i, T - 1) * H + 8 * q;
  const uint16_t* wrow[NE];
  rt_f32x16 acc[NE];
#pragma unroll
  for (int n = 0; n < NE; n++) {
    wrow[n] = wr + (int64_t)min(32 * n + i, E - 1) * H + 8 * q;
#pragma unroll
    for (int r = 0; r < 16; r++) acc[n][r] = 0.f;
  }
  for (int k = k0; k < k1; k += 16) {
    const rt_bf16x8 a = *(const rt_bf16x8*)(xrow + k);
#pragma unroll
    for (int n = 0; n < NE; n++) {
      const rt_bf16x8 b = *(const rt_bf16x8*)(wrow[n] + k);
      acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
    }
  }
  // the slices are added in wavefront order (fixed), tile by tile
#pragma unroll
  for (int n = 0; n < NE; n++) {
#pragma unroll
    for (int r = 0; r < 16; r++) part[wave][r * 64 + lane] = acc[n][r];
    __syncthreads();
    for (int idx = threadIdx.x; idx < 1024; idx += 64 * kRouterWaves) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < kRouterWaves; w++) s += part[w][idx];
      const int r = idx >> 6, l = idx & 63;
      const int e = 32 * n + (l & 31), t = t0 + (r % 4) + 4 * (l >> 5) + 8 * (r / 4);
      if (e < E && t < T) logits[(int64_t)t * E + e] = s;
    }
    __syncthreads();
  }
}

}  // namespace ssmm

extern "C" int ssmm_router_logits(const uint16_t* x, int T, int H, const uint16_t* wr, int E, float* logits,
                                  void* stream) {
  if (T < 0 || H < 1 || E < 1) return SSMM_EINVAL;
  if (H % 16 || E > kMaxExperts) return SSMM_ESHAPE;
  if (T == 0) return SSMM_OK;
  if (!x || !wr || !logits) return SSMM_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const dim3 grid((unsigned)((T + 31) / 32)), block(64 * kRouterWaves);
  const int ne = (E + 31) / 32;
  switch (ne) {
    case 1: hipLaunchKernelGGL(router_logits_kernel<1>, grid, block, 0, s, x, T, H, wr, E, logits); break;
    case 2: hipLaunchKernelGGL(router_logits_kernel<2>, grid, block, 0, s, x, T, H, wr, E, logits); break;
    case 3: hipLaunchKernelGGL(router_logits_kernel<3>, grid, block, 0, s, x, T, H, wr, E, logits); break;
    case 4: hipLaunchKernelGGL(router_logits_kernel<4>, grid, block, 0, s, x, T, H, wr, E, logits); break;
    case 5: hipLaunchKernelGGL(router_logits_kernel<5>, grid, block, 0, s, x, T, H, wr, E, logits); break;
    case 6: hipLaunchKernelGGL(router_logits_kernel<6>, grid, block, 0, s, x, T, H, wr, E, logits); break;
    case 7: hipLaunchKernelGGL(router_logits_kernel<7>, grid, block, 0, s, x, T, H, wr, E, logits); break;
    default: hipLaunchKernelGGL(router_logits_kernel<8>, grid, block, 0, s, x, T, H, wr, E, logits); break;
  }
  SSMM_RETURN_IF_LAUNCH_FAILED();
  return SSMM_OK;
}
