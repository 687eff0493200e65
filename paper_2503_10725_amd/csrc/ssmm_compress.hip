// Offline weight path: prune to the dual-side format and encode (section 4.1),
// decode, and the kernel-ready re-ordering and its inverse.
#include "ssmm_common.h"

namespace ssmm {

// ---------------------------------------------------------------------------
// Sub-Row selection: one thread per (expert, block row, segment).  The score of
// a Sub-Row is the fp64 sum of squares of its V values added in ascending
// column order (products of bf16 values are exact in fp64, so a fused multiply
// add rounds exactly as multiply-then-add does).  N rounds of "best not yet
// chosen", a strictly-greater compare keeping the lower row on ties.
// ---------------------------------------------------------------------------
__device__ inline double bf16_to_f64(uint16_t b) {
  return (double)__uint_as_float((uint32_t)b << 16);
}

__global__ void __launch_bounds__(256) select_subrows_kernel(const uint16_t* __restrict__ w, int64_t total,
                                                             int64_t rows, int64_t K, int N, int M, int V,
                                                             uint8_t* __restrict__ index) {
  int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (tid >= total) return;
  const int64_t segs = K / V, blocks = rows / M;
  const int64_t s = tid % segs, b = (tid / segs) % blocks, e = tid / (segs * blocks);
  const uint16_t* base = w + (e * rows + b * M) * K + s * V;
  uint64_t chosen[4] = {0, 0, 0, 0};
  for (int round = 0; round < N; round++) {
    int best = -1;
    double best_score = 0.0;
    for (int m = 0; m < M; m++) {
      if ((chosen[m >> 6] >> (m & 63)) & 1) continue;
      double score = 0.0;
      for (int v = 0; v < V; v++) {
        double x = bf16_to_f64(base[(int64_t)m * K + v]);
        score = score + x * x;
      }
      if (score != score) score = __builtin_huge_val();   // a Sub-Row with a NaN ranks like +infinity: it is kept, the NaN stays visible
      if (best < 0 || score > best_score) {
        best = m;
        best_score = score;
      }
    }
    chosen[best >> 6] |= (uint64_t)1 << (best & 63);
  }
  const int64_t rc = rows * N / M;
  int j = 0;
  for (int m = 0; m < M; m++)
    if ((chosen[m >> 6] >> (m & 63)) & 1) {
      index[(e * rc + b * N + j) * segs + s] = (uint8_t)m;
      j++;
    }
}

// 2:4 choice on one group: the two largest magnitudes, ties to the lower position.
// The order of |v| is the order of the bf16 bit pattern without its sign; a NaN ranks like an
// infinity (it is kept and stays visible in the outputs).
__device__ inline void choose_2of4(const uint16_t v[4], int& p0, int& p1) {
  int m[4];
  for (int i = 0; i < 4; i++) m[i] = min(v[i] & 0x7FFF, 0x7F80);
  int first = 0;
  for (int i = 1; i < 4; i++)
    if (m[i] > m[first]) first = i;
  int second = first == 0 ? 1 : 0;
  for (int i = 0; i < 4; i++)
    if (i != first && m[i] > m[second]) second = i;
  p0 = first < second ? first : second;
  p1 = first < second ? second : first;
}

// ---------------------------------------------------------------------------
// Encode: one thread per (expert, compressed row, 32-element chunk of K) = one
// metadata word, 8 groups, 16 kept values.  Writes the canonical arrays and,
// for plain 2:4, the kernel-ready form in the same pass.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) encode_kernel(const uint16_t* __restrict__ w, int64_t total, int64_t rows,
                                                     int64_t K, int N, int M, int V,
                                                     const uint8_t* __restrict__ index_in,
                                                     uint16_t* __restrict__ values, uint32_t* __restrict__ meta,
                                                     uint16_t* __restrict__ tiled_values,
                                                     uint16_t* __restrict__ tiled_meta,
                                                     uint8_t* __restrict__ tiled_vidx) {
  int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (tid >= total) return;
  const bool vec = N < M;
  const int64_t words = meta_words(K), rc = vec ? rows * N / M : rows;
  const int64_t wd = tid % words, r = (tid / words) % rc, e = tid / (words * rc);
  const int64_t groups = K / 4;
  uint16_t kept[16];
  uint32_t word = 0;
  int nib[8];
  for (int g8 = 0; g8 < 8; g8++) {
    const int64_t g = wd * 8 + g8;
    kept[2 * g8] = kept[2 * g8 + 1] = 0;
    nib[g8] = 0;
    if (g >= groups) continue;
    int64_t src_row = r;
    if (vec) {
      const int64_t s = (4 * g) / V;
      src_row = (r / N) * M + index_in[(e * rc + r) * (K / V) + s];
    }
    const uint16_t* p = w + (e * rows + src_row) * K + 4 * g;
    uint16_t v[4] = {p[0], p[1], p[2], p[3]};
    int p0, p1;
    choose_2of4(v, p0, p1);
    kept[2 * g8] = v[p0];
    kept[2 * g8 + 1] = v[p1];
    nib[g8] = p0 | (p1 << 2);
    word |= (uint32_t)nib[g8] << (4 * g8);
  }
  if (values) {
    uint16_t* dst = values + (e * rc + r) * (K / 2) + wd * 16;
    for (int g8 = 0; g8 < 8; g8++)
      if (wd * 8 + g8 < groups) {
        dst[2 * g8] = kept[2 * g8];
        dst[2 * g8 + 1] = kept[2 * g8 + 1];
      }
    meta[(e * rc + r) * words + wd] = word;
  }
  if (tiled_values) {  // rc % 32 == 0, K % 64 == 0: wd is the k block
    const int64_t MT = rc / 32, KB = K / 32;
    const int64_t mt = r / 32;
    const int i = rowmap_inv((int)(r % 32));
    for (int q = 0; q < 2; q++) {
      const int lane = 32 * q + i;
      uint16_t* dst = tiled_values + (((e * MT + mt) * KB + wd) * 64 + lane) * 8;
      uint32_t idx16 = 0;
      for (int G = 0; G < 8; G++) {
        if (group_lane_half(G) != q) continue;
        const int g = group_slot_pair(G);
        dst[2 * g] = kept[2 * G];
        dst[2 * g + 1] = kept[2 * G + 1];
        idx16 |= (uint32_t)nib[G] << (4 * g);
      }
      const int64_t slot = ((((e * MT + mt) * (KB / 2) + wd / 2) * 64 + lane) << 1) + (wd & 1);
      tiled_meta[slot] = (uint16_t)idx16;
      if (tiled_vidx) {  // (1,2,V), V % 8 == 0: which dense row the lane's two 8-element segments of this k block came from
        const uint8_t* ix = index_in + (e * rc + r) * (K / V);
        tiled_vidx[slot] = (uint8_t)(ix[(32 * wd + 8 * q) / V] | (ix[(32 * wd + 8 * (2 + q)) / V] << 1));
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Decode: one thread per (expert, dense row, 32-element chunk of K); writes all
// 32 elements, zeros included, so the destination needs no clearing.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) decode_kernel(const uint16_t* __restrict__ values,
                                                     const uint32_t* __restrict__ meta,
                                                     const uint8_t* __restrict__ index, int64_t total, int64_t rows,
                                                     int64_t K, int N, int M, int V, uint16_t* __restrict__ out) {
  int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (tid >= total) return;
  const bool vec = N < M;
  const int64_t words = meta_words(K), rc = vec ? rows * N / M : rows;
  const int64_t wd = tid % words, r = (tid / words) % rows, e = tid / (words * rows);
  const int64_t groups = K / 4;
  for (int g8 = 0; g8 < 8; g8++) {
    const int64_t g = wd * 8 + g8;
    if (g >= groups) break;
    int64_t cr = r;
    bool live = true;
    if (vec) {
      const int64_t s = (4 * g) / V, b = r / M;
      const int off = (int)(r % M);
      live = false;
      for (int j = 0; j < N; j++)
        if (index[(e * rc + b * N + j) * (K / V) + s] == off) {
          live = true;
          cr = b * N + j;
        }
    }
    uint16_t o[4] = {0, 0, 0, 0};
    if (live) {
      const uint32_t word = meta[(e * rc + cr) * words + wd];
      const int nb = (word >> (4 * g8)) & 0xF;
      const uint16_t* v = values + (e * rc + cr) * (K / 2) + 2 * g;
      o[nb & 3] = v[0];
      o[nb >> 2] = v[1];
    }
    uint16_t* dst = out + (e * rows + r) * K + 4 * g;
    for (int i = 0; i < 4; i++) dst[i] = o[i];
  }
}

// Kernel-ready form -> canonical arrays (plain 2:4): exact inverse of the tiled
// branch of encode_kernel.  One thread per (expert, row, k block).
__global__ void __launch_bounds__(256) untile_kernel(const uint16_t* __restrict__ tiled_values,
                                                     const uint16_t* __restrict__ tiled_meta,
                                                     const uint8_t* __restrict__ tiled_vidx, int64_t total,
                                                     int64_t rc, int64_t K, int V, uint16_t* __restrict__ values,
                                                     uint32_t* __restrict__ meta, uint8_t* __restrict__ index) {
  int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (tid >= total) return;
  const int64_t KB = K / 32, MT = rc / 32;
  const int64_t kb = tid % KB, r = (tid / KB) % rc, e = tid / (KB * rc);
  const int64_t mt = r / 32;
  const int i = rowmap_inv((int)(r % 32));
  uint32_t word = 0;
  uint16_t* dst = values + (e * rc + r) * (K / 2) + kb * 16;
  for (int G = 0; G < 8; G++) {
    const int lane = 32 * group_lane_half(G) + i, g = group_slot_pair(G);
    const uint16_t* src = tiled_values + (((e * MT + mt) * KB + kb) * 64 + lane) * 8;
    dst[2 * G] = src[2 * g];
    dst[2 * G + 1] = src[2 * g + 1];
    const uint32_t idx16 = tiled_meta[((((e * MT + mt) * (KB / 2) + kb / 2) * 64 + lane) << 1) + (kb & 1)];
    word |= ((idx16 >> (4 * g)) & 0xF) << (4 * G);
  }
  if (tiled_vidx)
    for (int q = 0; q < 2; q++) {
      const uint8_t b = tiled_vidx[((((e * MT + mt) * (KB / 2) + kb / 2) * 64 + 32 * q + i) << 1) + (kb & 1)];
      uint8_t* ix = index + (e * rc + r) * (K / V);
      const int64_t k0 = 32 * kb + 8 * q, k1 = 32 * kb + 8 * (2 + q);   // the Sub-Row's first 8 elements carry its index
      if (k0 % V == 0) ix[k0 / V] = b & 1;
      if (k1 % V == 0) ix[k1 / V] = (b >> 1) & 1;
    }
  meta[(e * rc + r) * KB + kb] = word;
}

// Gathered formats: the third section of the kernel-ready form.  One thread per (expert, dense
// row, k block): the stored Sub-Row (if any) that holds this dense row's values in the k block.
__global__ void __launch_bounds__(256) gather_index_kernel(const uint8_t* __restrict__ index, int64_t total, int64_t rows,
                                                           int64_t K, int N, int M, int V, uint8_t* __restrict__ tiled_vidx) {
  int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (tid >= total) return;
  const int64_t KB = K / 32, rc = rows * N / M;
  const int64_t kb = tid % KB, R = (tid / KB) % rows, e = tid / (KB * rows);
  const int64_t b = R / M, s = 32 * kb / V;
  const int off = (int)(R % M);
  uint8_t d = 0x80;
  for (int j = 0; j < N; j++)
    if (index[(e * rc + b * N + j) * (K / V) + s] == off) d = (uint8_t)rowmap_inv((int)((b * N + j) % 32));
  const int i = rowmap_inv((int)(R % 32));
  tiled_vidx[(((e * (rows / 32) + R / 32) * (KB / 2) + kb / 2) * 32 + i) * 2 + (kb & 1)] = d;
}
// ... and back: one thread per (expert, stored row, Sub-Row position): the dense row of its block
// whose entry points at this stored row.
__global__ void __launch_bounds__(256) ungather_index_kernel(const uint8_t* __restrict__ tiled_vidx, int64_t total,
                                                             int64_t rows, int64_t K, int N, int M, int V,
                                                             uint8_t* __restrict__ index) {
  int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (tid >= total) return;
  const int64_t KB = K / 32, rc = rows * N / M, S = K / V;
  const int64_t s = tid % S, c = (tid / S) % rc, e = tid / (S * rc);
  const int64_t b = c / N, kb = s * V / 32;
  const uint8_t want = (uint8_t)rowmap_inv((int)(c % 32));
  uint8_t found = 0;
  for (int off = 0; off < M; off++) {
    const int64_t R = b * M + off;
    const int i = rowmap_inv((int)(R % 32));
    if (tiled_vidx[(((e * (rows / 32) + R / 32) * (KB / 2) + kb / 2) * 32 + i) * 2 + (kb & 1)] == want) found = (uint8_t)off;
  }
  index[(e * rc + c) * S + s] = found;
}

inline unsigned grid_for(int64_t total) { return (unsigned)((total + 255) / 256); }

}  // namespace ssmm

using namespace ssmm;

extern "C" const char* ssmm_strerror(int status) {
  switch (status) {
    case SSMM_OK: return "ok";
    case SSMM_EINVAL: return "invalid argument (null pointer or scalar out of range)";
    case SSMM_ESHAPE: return "shape not admitted by the format or the kernels";
    case SSMM_EWORKSPACE: return "workspace too small";
    case SSMM_EHIP: return "HIP runtime error at launch";
    case SSMM_ELIMIT: return "size beyond the fixed scratch of an entry point that takes no workspace";
    default: return "unknown status";
  }
}

extern "C" int ssmm_compressed_sizes(int64_t rows, int64_t K, ssmm_format f, size_t* values_bytes,
                                     size_t* meta_bytes, size_t* index_bytes, size_t* tiled_bytes) {
  int st = check_format(f, rows, K);
  if (st) return st;
  const int64_t rc = compressed_rows(f, rows);
  const size_t vb = (size_t)rc * (K / 2) * 2, mb = (size_t)rc * meta_words(K) * 4;
  if (values_bytes) *values_bytes = vb;
  if (meta_bytes) *meta_bytes = mb;
  if (index_bytes) *index_bytes = is_vectorwise(f) ? (size_t)rc * (K / f.V) : 0;
  if (tiled_bytes) *tiled_bytes = can_tile(f, rows, K) ? vb + mb + tiled_vidx_bytes(f, rc, K) : 0;
  return SSMM_OK;
}

extern "C" int ssmm_compress_weights(const uint16_t* w_dense, int E, int64_t rows, int64_t K, ssmm_format f,
                                     uint16_t* values, uint32_t* meta, uint8_t* index, void* tiled,
                                     void* stream) {
  if (E < 0) return SSMM_EINVAL;
  int st = check_format(f, rows, K);
  if (st) return st;
  if (E == 0) return SSMM_OK;   // nothing to encode; pointers may be null
  if (!w_dense) return SSMM_EINVAL;
  const bool vec = is_vectorwise(f);
  const bool canonical = values != nullptr;
  if (canonical && (!meta || (vec && !index))) return SSMM_EINVAL;
  if (!canonical && (meta || !tiled)) return SSMM_EINVAL;
  if (tiled && !can_tile(f, rows, K)) return SSMM_ESHAPE;
  if (vec && !canonical) return SSMM_EINVAL;  // the Sub-Row choice needs the index array as its store
  hipStream_t s = (hipStream_t)stream;
  const int64_t rc = compressed_rows(f, rows);
  if (vec) {
    const int64_t total = (int64_t)E * (rows / f.M) * (K / f.V);
    hipLaunchKernelGGL(select_subrows_kernel, dim3(grid_for(total)), dim3(256), 0, s, w_dense, total, rows, K, f.N,
                       f.M, f.V, index);
    SSMM_RETURN_IF_LAUNCH_FAILED();
  }
  uint16_t* tv = (uint16_t*)tiled;
  uint16_t* tm = tiled ? tv + (size_t)E * rc * (K / 2) : nullptr;
  uint8_t* tx = (tiled && vec) ? (uint8_t*)tiled + E * (tiled_values_bytes(rc, K) + tiled_meta_bytes(rc, K)) : nullptr;
  const int64_t total = (int64_t)E * rc * meta_words(K);
  const bool gathered = gathered_format(f);
  hipLaunchKernelGGL(encode_kernel, dim3(grid_for(total)), dim3(256), 0, s, w_dense, total, rows, K, f.N, f.M, f.V,
                     (const uint8_t*)index, values, meta, tv, tm, gathered ? nullptr : tx);
  SSMM_RETURN_IF_LAUNCH_FAILED();
  if (tiled && gathered) {
    const int64_t n = (int64_t)E * rows * (K / 32);
    hipLaunchKernelGGL(gather_index_kernel, dim3(grid_for(n)), dim3(256), 0, s, (const uint8_t*)index, n, rows, K, f.N, f.M,
                       f.V, tx);
    SSMM_RETURN_IF_LAUNCH_FAILED();
  }
  return SSMM_OK;
}

extern "C" int ssmm_decompress_weights(const uint16_t* values, const uint32_t* meta, const uint8_t* index, int E,
                                       int64_t rows, int64_t K, ssmm_format f, uint16_t* w_dense_out,
                                       void* stream) {
  if (!values || !meta || !w_dense_out || E < 0) return SSMM_EINVAL;
  int st = check_format(f, rows, K);
  if (st) return st;
  if (is_vectorwise(f) && !index) return SSMM_EINVAL;
  if (E == 0) return SSMM_OK;
  const int64_t total = (int64_t)E * rows * meta_words(K);
  hipLaunchKernelGGL(decode_kernel, dim3(grid_for(total)), dim3(256), 0, (hipStream_t)stream, values, meta, index,
                     total, rows, K, f.N, f.M, f.V, w_dense_out);
  SSMM_RETURN_IF_LAUNCH_FAILED();
  return SSMM_OK;
}

extern "C" int ssmm_untile_weights(const void* tiled, int E, int64_t rows, int64_t K, ssmm_format f,
                                   uint16_t* values, uint32_t* meta, uint8_t* index, void* stream) {
  if (!tiled || !values || !meta || E < 0) return SSMM_EINVAL;
  int st = check_format(f, rows, K);
  if (st) return st;
  if (!can_tile(f, rows, K)) return SSMM_ESHAPE;
  if (is_vectorwise(f) && !index) return SSMM_EINVAL;
  if (E == 0) return SSMM_OK;
  const int64_t rc = compressed_rows(f, rows);
  const uint16_t* tv = (const uint16_t*)tiled;
  const uint16_t* tm = tv + (size_t)E * rc * (K / 2);
  const uint8_t* tx = is_vectorwise(f)
                          ? (const uint8_t*)tiled + E * (tiled_values_bytes(rc, K) + tiled_meta_bytes(rc, K))
                          : nullptr;
  const int64_t total = (int64_t)E * rc * (K / 32);
  const bool gathered = gathered_format(f);
  hipLaunchKernelGGL(untile_kernel, dim3(grid_for(total)), dim3(256), 0, (hipStream_t)stream, tv, tm, gathered ? nullptr : tx,
                     total, rc, K, is_vectorwise(f) ? f.V : 8, values, meta, index);
  SSMM_RETURN_IF_LAUNCH_FAILED();
  if (gathered) {
    const int64_t n = (int64_t)E * rc * (K / f.V);
    hipLaunchKernelGGL(ungather_index_kernel, dim3(grid_for(n)), dim3(256), 0, (hipStream_t)stream, tx, n, rows, K, f.N, f.M,
                       f.V, index);
    SSMM_RETURN_IF_LAUNCH_FAILED();
  }
  return SSMM_OK;
}
