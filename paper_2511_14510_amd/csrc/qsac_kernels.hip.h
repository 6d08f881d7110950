// Device code of the QSAC decode step for gfx950 (CDNA4, 64-wide wavefronts).
//
// Stages, in launch order (one iteration of Algorithm 1 of the LiteCache paper for every
// (batch, KV head) pair p at once):
//   gate     cache lookup: CosSim (Section 3.1) per query head in fp64, Eq. (2) per KV head,
//            label update q_c <- q_t on a miss (the paper fuses the two as well, Section 6.2)
//   score    Eq. (1) for the head's query group against all N keys, S[n] = max_g q_g.k_n,
//            stored as order-preserving 32-bit keys
//   select   radix select of the k-th largest key (11 + 11 + 10 bits), ties by lowest index,
//            ascending index list, hit mask against the cached tokens, (slot, token) miss
//            list, slot table update.  Up to kSmallMaxN keys: one workgroup per pair does all
//            of it with its bitmaps in LDS (above 16384 keys on a candidate list cut out by a
//            sampled bound).  Beyond: the first histogram is fused into the scoring kernel and
//            the levels run as grid-wide kernels (refine1, refine2, mark) so that a few pairs
//            with very long contexts still fill the chip, followed by the one-workgroup diff
//            on the bitmaps, or, above 262144 keys, by a grid-wide emit of the set as a token
//            list and a one-workgroup diff on that list.
//   fill     copies the missing K / V rows from the fill sources into the slots; by default this
//            is folded into the attention kernel's row loads ("fill on read"), the separate
//            kernel (optionally on a side stream) is kept as the alternative
//   attn     softmax(q K_c^T / sqrt(d)) V_c over the slots (Section 2.1), split over slots
//   combine  merges the splits
//
// Pairs whose gate reused the cache leave every miss-path kernel at once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qsac {

typedef uint32_t u32;
typedef unsigned long long u64;

constexpr int kD = 128;            // head_dim
constexpr int kRowU4 = 16;         // 16-byte chunks per 256-byte row
constexpr int kBins = 2048;        // bins per radix level (level 2 uses the first 1024)
constexpr int kHistCopies = 4;     // one-workgroup select: lane l counts into copy l % 4 (fewer same-address conflicts)
constexpr int kCandBins = 4096;    // one-workgroup select, guided path: bins of the candidates' histogram,
constexpr int kCandShift = 13;     // each 2^kCandShift keys wide
constexpr int kHistPitch = kBins + 16;  // words between copies: the same bin of different copies sits in different banks
static_assert(4096 + kCandBins <= kHistCopies * kHistPitch && kCandBins <= 8 * 1024,
              "the candidates' level sits behind the sample's 4096 bins in the one-workgroup select's histogram");
constexpr int kScoreRowsSmall = 256;   // keys per workgroup of the scoring kernel (small-N path)
constexpr int kScoreRowsLarge = 1024;  // ... when the level-0 histogram is fused in (large-N path)
constexpr int kSmallMaxN = 65536;      // largest N the one-workgroup select takes: its keys fit in the registers of 1024 threads
constexpr int kTilePitch = 272;        // bytes between key rows of an LDS tile: 256 + 16 keeps b128 reads conflict-free
constexpr int kSelChunk = 8192;    // keys per workgroup of the select passes
constexpr int kFillRows = 64;      // miss-list entries per workgroup of the fill kernel
constexpr int kDiffThreads = 1024;
constexpr int kSelectListCap = 8192;   // candidates the guided select can hold in LDS (64 KiB of keys + indices)

typedef __attribute__((ext_vector_type(2))) _Float16 half2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf2_t;
typedef __attribute__((ext_vector_type(8))) _Float16 half8_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf8_t;
typedef __attribute__((ext_vector_type(4))) float f4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t v4u;  // one 16-byte load

struct TauArg {
  float v[64];  // per KV head
};

// Where the K / V rows of a pair's missing tokens come from.  A resident KV head (Section 4.4 of
// the paper: heads that are hard to reuse keep their full KV in HBM) takes K rows from the HBM
// copy of K that scoring reads and V rows from the resident V tensor [B, n_res, N, D]; the others
// take both from the fill sources (HBM or host-mapped pinned memory), [B, Hkv, N, D].
struct FillSrc {
  const v4u* K_src;
  const v4u* V_src;
  const v4u* K_res;
  const v4u* V_res;
  int n_res;
  int host_row_bytes;    // bytes of a (K row, V row) pair of a non-resident head that come from host memory: 0, 256 or 512
  signed char slot[64];  // per KV head: index in V_res, -1 if not resident
};

// Per-step scalars read from device memory when a step is replayed from a captured graph (mirror of
// qsac_dev_params in qsac.h).
struct DevParams {
  float tau[64];
  int n_app;
  int reserved[3];
};
__device__ __forceinline__ void fill_rows_of(const FillSrc& f, int p, int Hkv, int64_t N, const v4u*& Ks,
                                             const v4u*& Vs) {
  const int b = p / Hkv, h = p % Hkv;
  const int rs = f.slot[h];
  if (rs >= 0) {
    Ks = f.K_res + (size_t)p * (size_t)N * kRowU4;
    Vs = f.V_res + ((size_t)b * f.n_res + rs) * (size_t)N * kRowU4;
  } else {
    Ks = f.K_src + (size_t)p * (size_t)N * kRowU4;
    Vs = f.V_src + (size_t)p * (size_t)N * kRowU4;
  }
}

// ---------------------------------------------------------------- small helpers

__device__ __forceinline__ u32 fbits(float f) { return __builtin_bit_cast(u32, f); }
__device__ __forceinline__ float bitsf(u32 u) { return __builtin_bit_cast(float, u); }

// Key of a token at position n of N: sink tokens (the first n_sink) and recent tokens (the last
// n_recent) are kept in the cache persistently (Section 7.1 of the paper), i.e. they rank above
// every score; positions at and past N get key 0, below every score.
__device__ __forceinline__ u32 ordered_key(float f);
__device__ __forceinline__ u32 token_key(float score, int64_t n, int64_t N, int n_sink, int n_recent) {
  if (n >= N) return 0u;
  if (n < n_sink || n >= N - n_recent) return 0xffffffffu;
  return ordered_key(score);
}

// Order-preserving image of a finite fp32: a > b  <=>  key(a) > key(b); -0 ranks as +0.
__device__ __forceinline__ u32 ordered_key(float f) {
  u32 u = fbits(f);
  if ((u << 1) == 0) u = 0;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int DT>
__device__ __forceinline__ float lo16(u32 w) {
  if (DT == 0) return (float)__builtin_bit_cast(half2_t, w)[0];
  return bitsf(w << 16);
}
template <int DT>
__device__ __forceinline__ float hi16(u32 w) {
  if (DT == 0) return (float)__builtin_bit_cast(half2_t, w)[1];
  return bitsf(w & 0xffff0000u);
}

template <int DT>
__device__ __forceinline__ float dot2(u32 a, u32 b, float acc) {
  if (DT == 0) return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), acc, false);
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2_t, a), __builtin_bit_cast(bf2_t, b), acc, false);
}
template <int DT>
__device__ __forceinline__ float dot8(v4u a, v4u b) {
  float s = dot2<DT>(a.x, b.x, 0.f);
  s = dot2<DT>(a.y, b.y, s);
  s = dot2<DT>(a.z, b.z, s);
  return dot2<DT>(a.w, b.w, s);
}

template <int DT>
__device__ __forceinline__ f4_t mfma16(v4u a, v4u b, f4_t c) {
  if (DT == 0) return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8_t, a), __builtin_bit_cast(bf8_t, b), c, 0, 0, 0);
}

// Sum over the 16 lanes of a DPP row; every lane of the row ends with the same total.
// All 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return bitsf((u32)__builtin_amdgcn_update_dpp(0, (int)fbits(v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);  // row_half_mirror
  v += dpp_move<0x140>(v);  // row_mirror
  return v;
}

// Inclusive prefix sum over the 64 lanes of a wave, in DPP: Kogge-Stone inside each row of 16
// (row_shr 1, 2, 4, 8, zero-filled), then lane 15 of row 0 / 2 into rows 1 / 3, then lane 31 into
// rows 2 and 3.  All 64 lanes must be active.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
  return v;
}

// Sum of a double over the 64 lanes of a wave, delivered in lane 63 (other lanes hold partial
// prefixes).  Same DPP ladder as wave_inclusive_scan, applied to both halves of the value.
template <int CTRL, int ROW_MASK, bool BOUND>
__device__ __forceinline__ double dpp_f64(double v) {
  const unsigned long long u = __builtin_bit_cast(unsigned long long, v);
  const u32 lo = (u32)__builtin_amdgcn_update_dpp(0, (int)(u32)u, CTRL, ROW_MASK, 0xf, BOUND);
  const u32 hi = (u32)__builtin_amdgcn_update_dpp(0, (int)(u32)(u >> 32), CTRL, ROW_MASK, 0xf, BOUND);
  return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);  // masked-off rows read +0.0
}
__device__ __forceinline__ double wave_sum_f64_lane63(double v) {
  v += dpp_f64<0x111, 0xf, true>(v);
  v += dpp_f64<0x112, 0xf, true>(v);
  v += dpp_f64<0x114, 0xf, true>(v);
  v += dpp_f64<0x118, 0xf, true>(v);
  v += dpp_f64<0x142, 0xa, false>(v);
  v += dpp_f64<0x143, 0xc, false>(v);
  return v;
}

// Clears `words` 32-bit words of LDS at p (16-byte aligned) with 16-byte stores; NT threads.
template <int NT>
__device__ __forceinline__ void lds_zero(u32* p, int words) {
  v4u* p4 = reinterpret_cast<v4u*>(p);
  const int n4 = words >> 2;
  for (int i = threadIdx.x; i < n4; i += NT) p4[i] = v4u{0, 0, 0, 0};
  if ((int)threadIdx.x < (words & 3)) p[(n4 << 2) + threadIdx.x] = 0;
}

// Sum of v over lanes 0..15 of the wave, returned as a wave-uniform value (Kogge-Stone over DPP row 0, then
// a read of lane 15).  All 64 lanes must be active.
__device__ __forceinline__ int row0_total(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);
  return __builtin_amdgcn_readlane(v, 15);
}

// The per-wave values of a workgroup of NW <= 16 wavefronts sit in s[0..NW): returns the sum of the values of
// the waves below this one; *total gets the sum of all.  Lane l reads s[l] and the sums are taken across lanes.
template <int NW>
__device__ __forceinline__ int below_and_total(const int* s, int* total) {
  static_assert(NW <= 16, "one DPP row holds the per-wave values");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = lane < NW ? s[lane] : 0;
  if (total) *total = row0_total(t);
  return row0_total(lane < wave ? t : 0);
}

// Exclusive prefix sum of one int per thread over a workgroup of NW wavefronts; *total gets the sum.
// Contains barriers: every thread of the workgroup must call it.
template <int NW>
__device__ __forceinline__ int block_exclusive_scan(int v, int* s_wave /*[NW]*/, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int inc = wave_inclusive_scan(v);
  __syncthreads();  // s_wave may still be read from a previous call
  if (lane == 63) s_wave[wave] = inc;
  __syncthreads();
  return below_and_total<NW>(s_wave, total) + inc - v;
}

// Exclusive prefix over the waves of a workgroup of one value per wave (the same in all its lanes).
// Contains barriers.
template <int NW>
__device__ __forceinline__ int wave_totals_exclusive(int wave_value, int* s_wave, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) s_wave[wave] = wave_value;
  __syncthreads();
  return below_and_total<NW>(s_wave, total);
}

// The same for three values per wave at once (s_wave3: 3 * NW ints); *total_c gets the sum of the third.
// LEAD = false: a barrier already separates the call from the last use of s_wave3.
template <int NW, bool LEAD = true>
__device__ __forceinline__ void wave_totals_exclusive3(int va, int vb, int vc, int* s_wave3 /*[3*NW]*/, int* base_a,
                                                       int* base_b, int* base_c, int* total_c) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (LEAD) __syncthreads();
  if (lane == 0) {
    s_wave3[wave] = va;
    s_wave3[NW + wave] = vb;
    s_wave3[2 * NW + wave] = vc;
  }
  __syncthreads();
  *base_a = below_and_total<NW>(s_wave3, nullptr);
  *base_b = below_and_total<NW>(s_wave3 + NW, nullptr);
  *base_c = below_and_total<NW>(s_wave3 + 2 * NW, total_c);
}

// Among bins [0, nbins) of `hist`, finds the bin b with  count(bins > b) < need <= count(bins >= b).
// Returns b and *above = count(bins > b), or -1 if the bins hold fewer than `need` in all; *total (optional)
// gets the sum of all bins, *in_bin (optional; s_res then has three words) the count of bin b.  NT threads (nbins is a multiple of NT, at most 8 bins per thread); the histogram
// (16-byte aligned) may be split over COPIES copies kHistPitch words apart.  Contains two barriers; the caller's barrier that
// publishes the histogram must also be the last thing before the call that touched s_wave and s_res.
template <int NT, int COPIES = 1>
__device__ __forceinline__ int find_bin(const u32* hist, int nbins, int need, int* above, int* s_wave,
                                        int* s_res, int* total = nullptr, int* in_bin = nullptr) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int per = nbins / NT;
  // thread t owns bins [hi - per + 1, hi] counted from the top: t = 0 owns the highest bins
  const int hi = nbins - 1 - (int)threadIdx.x * per;
  int c[8];
  int local = 0;
  if (COPIES == 1 && per == 4) {  // hist is 16-byte aligned: the four bins in one read
    const v4u q = *reinterpret_cast<const v4u*>(hist + hi - 3);
    c[0] = (int)q.w, c[1] = (int)q.z, c[2] = (int)q.y, c[3] = (int)q.x;
    c[4] = c[5] = c[6] = c[7] = 0;
    local = c[0] + c[1] + c[2] + c[3];
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      c[i] = 0;
      if (i < per) {
#pragma unroll
        for (int cp = 0; cp < COPIES; ++cp) c[i] += (int)hist[cp * kHistPitch + hi - i];
      }
      local += c[i];
    }
  }
  const int inc = wave_inclusive_scan(local);
  if (lane == 63) s_wave[wave] = inc;
  __syncthreads();
  int tot;
  const int before = below_and_total<NT / 64>(s_wave, &tot) + inc - local;  // keys in bins above this thread's
  if (total) *total = tot;
  if (before < need && need <= before + local) {
    int run = before;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (i < per) {
        if (run < need && need <= run + c[i]) {
          s_res[0] = hi - i;
          s_res[1] = run;
          if (in_bin) s_res[2] = c[i];
        }
        run += c[i];
      }
    }
  }
  __syncthreads();
  if (need > tot) return -1;
  *above = s_res[1];
  if (in_bin) *in_bin = s_res[2];
  return s_res[0];
}

// ---------------------------------------------------------------- gate

// One workgroup (256 threads) per pair.  Wave w takes query heads w, w+4, ...; each lane two
// elements.  The three dot products, the norms and Eq. (2) are taken in fp64: products of two
// 16-bit floats are exact there, so the reuse decision matches an fp64 reference unless the
// aggregate sits within ~1e-15 of tau.
template <int DT>
__global__ __launch_bounds__(256) void qsac_gate_kernel(
    const uint16_t* __restrict__ q, uint16_t* __restrict__ prev_q, const double* __restrict__ importance,
    TauArg tau, const u32* __restrict__ valid, const int* __restrict__ set_sorted, int* __restrict__ topk_idx,
    uint8_t* __restrict__ hit_mask, uint8_t* __restrict__ reuse_flags, float* __restrict__ sim_out,
    int* __restrict__ miss_count, u32* __restrict__ hist, u64* __restrict__ stats, int Hq, int Hkv, int G,
    int k, int k_max, bool clear_hist, const DevParams* __restrict__ dp) {
  const int p = blockIdx.x;
  const int b = p / Hkv, h = p % Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __shared__ double s_sim[8];
  __shared__ double s_imp[8];
  __shared__ int s_reuse;
  const size_t head0 = (size_t)b * Hq + (size_t)h * G;
  const u32* q32 = reinterpret_cast<const u32*>(q) + head0 * (kD / 2);
  u32* pq32 = reinterpret_cast<u32*>(prev_q) + head0 * (kD / 2);
  // everything the decision needs is requested up front, so the kernel pays one memory round trip
  const u32 was_valid = valid[p];
  const float tau_h = dp ? dp->tau[h] : tau.v[h];
  if (threadIdx.x < G) s_imp[threadIdx.x] = importance[h * G + threadIdx.x];

  for (int g = wave; g < G; g += 4) {
    u32 a = q32[g * 64 + lane], c = pq32[g * 64 + lane];
    double a0 = (double)lo16<DT>(a), a1 = (double)hi16<DT>(a);
    double c0 = (double)lo16<DT>(c), c1 = (double)hi16<DT>(c);
    double ab = a0 * c0 + a1 * c1, aa = a0 * a0 + a1 * a1, cc = c0 * c0 + c1 * c1;
    ab = wave_sum_f64_lane63(ab);
    aa = wave_sum_f64_lane63(aa);
    cc = wave_sum_f64_lane63(cc);
    if (lane == 63) {
      double s = (aa == 0.0 || cc == 0.0) ? -1.0 : ab / (sqrt(aa) * sqrt(cc));
      s_sim[g] = s;
      if (sim_out) sim_out[head0 + g] = (float)s;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double num = 0.0, den = 0.0;
    bool nonpos = false;
    for (int g = 0; g < G; ++g) {
      double w = s_imp[g];
      double s = s_sim[g];
      if (s <= 0.0) nonpos = true;
      num += w;
      den += w / s;
    }
    double agg = nonpos ? -1.0 : num / den;
    int reuse = (was_valid != 0) && (agg >= (double)tau_h);
    s_reuse = reuse;
    reuse_flags[p] = (uint8_t)reuse;
    atomicAdd(&stats[reuse ? 1 : 2], 1ull);
  }
  __syncthreads();
  if (s_reuse) {
    // cache hit: the cached set is reported as it stands by report_cached_set, in the select's launch,
    // where it costs nothing (the pairs that missed keep that launch busy far longer)
    if (threadIdx.x == 0) miss_count[p] = 0;
  } else {
    // cache miss: relabel now (the rows follow in the fill), and clear this pair's histograms
    // (only the grid-wide select uses them)
    for (int i = threadIdx.x; i < G * 64; i += 256) pq32[i] = q32[i];
    if (clear_hist) {
      u32* hp = hist + (size_t)p * 3 * kBins;
      for (int i = threadIdx.x; i < 3 * kBins; i += 256) hp[i] = 0;
    }
  }
}

// Cache hit: topk_idx <- the cached set (ascending), hit_mask <- 1.  Called by the workgroup that
// would have selected for the pair had it missed.
__device__ __forceinline__ void report_cached_set(const int* __restrict__ set_sorted, int* __restrict__ topk_idx,
                                                  uint8_t* __restrict__ hit_mask, int p, int k, int k_max) {
  const int* src = set_sorted + (size_t)p * k_max;
  for (int j = threadIdx.x; j < k; j += blockDim.x) {
    topk_idx[(size_t)p * k + j] = src[j];
    hit_mask[(size_t)p * k + j] = 1;
  }
}

// ---------------------------------------------------------------- score

// Large-N path only: after the key tile of a workgroup sits in LDS, write it out and add it to
// the pair's level-0 histogram.
__device__ __forceinline__ void score_hist_epilogue(const u32* s_keys, u32* s_hist, u32* __restrict__ keys_p,
                                                    u32* __restrict__ hist_p, int64_t row0, int64_t N) {
  __syncthreads();
  const int t4 = threadIdx.x * 4;
  v4u kk = *reinterpret_cast<const v4u*>(s_keys + t4);
  *reinterpret_cast<v4u*>(keys_p + row0 + t4) = kk;
  const int64_t n = row0 + t4;
  if (n + 0 < N) atomicAdd(&s_hist[kk.x >> 21], 1u);
  if (n + 1 < N) atomicAdd(&s_hist[kk.y >> 21], 1u);
  if (n + 2 < N) atomicAdd(&s_hist[kk.z >> 21], 1u);
  if (n + 3 < N) atomicAdd(&s_hist[kk.w >> 21], 1u);
  __syncthreads();
  for (int bin = threadIdx.x; bin < kBins; bin += 256) {
    u32 c = s_hist[bin];
    if (c) atomicAdd(&hist_p[bin], c);
  }
}

// MFMA form.  Per wave and 16-key tile, the 16 x 128 block of K meets the query group (zero
// padded to 16 rows) in four v_mfma_f32_16x16x32: queries are the A operand (row = query),
// keys the B operand (column = key); acc[i] of lane l is the score of query 4*(l/16)+i against
// key l%16.  The B operand wants lane l to hold pieces of key row l%16, which read straight
// from HBM costs half the bandwidth (every load instruction touches 32 cache lines for 1 KiB).
// So each wave reads its tile with four fully coalesced 1-KiB loads (lane l: 16 bytes at
// l*16), parks it in a wave-private LDS tile with a 272-byte row pitch, and reads the operand
// layout back from there, conflict-free.  Sixteen global loads per lane are in flight before
// the first tile is consumed.  Both operands are cut into the same 8-element pieces, so the
// products pair up correctly whatever order the hardware sums them in.
// ROWS keys per workgroup (four waves, ROWS/4 each).  HIST fuses the level-0 histogram.
template <int DT, int G, int ROWS, bool HIST>
__global__ __launch_bounds__(256) void qsac_score_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint8_t* __restrict__ reuse_flags,
    u32* __restrict__ keys, u32* __restrict__ hist, int Hq, int Hkv, int64_t N, int64_t n_pad, int n_sink,
    int n_recent) {
  const int p = blockIdx.y;
  if (reuse_flags[p]) return;
  __shared__ __attribute__((aligned(16))) unsigned char s_tile[4][2][16 * kTilePitch];
  __shared__ u32 s_hist[HIST ? kBins : 1];
  __shared__ __attribute__((aligned(16))) u32 s_keys[HIST ? ROWS : 4];
  if (HIST)
    for (int i = threadIdx.x; i < kBins; i += 256) s_hist[i] = 0;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = lane & 15, quarter = lane >> 4;
  const int b = p / Hkv, h = p % Hkv;
  const v4u* qg = reinterpret_cast<const v4u*>(q + ((size_t)b * Hq + (size_t)h * G) * kD);
  v4u qa[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) qa[j] = (m < G) ? qg[m * kRowU4 + quarter * 4 + j] : v4u{0, 0, 0, 0};

  const int64_t row0 = (int64_t)blockIdx.x * ROWS;
  const v4u* Kp = reinterpret_cast<const v4u*>(K + (size_t)p * (size_t)N * kD);
  constexpr int WROWS = ROWS / 4;
  const int wrow = wave * WROWS;
  u32* kout = keys + (size_t)p * n_pad + row0;
  const int64_t last = N - 1;

  for (int t0 = 0; t0 < WROWS / 16; t0 += 4) {
    v4u g[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t tile_row = row0 + wrow + (t0 + u) * 16;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int64_t n = tile_row + 4 * j + quarter;  // lane l: row 4j + l/16 of the tile, piece l%16
        n = n < last ? n : last;
        g[u][j] = __builtin_nontemporal_load(Kp + n * kRowU4 + m);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      unsigned char* tile = s_tile[wave][u & 1];
#pragma unroll
      for (int j = 0; j < 4; ++j)
        *reinterpret_cast<v4u*>(tile + (4 * j + quarter) * kTilePitch + m * 16) = g[u][j];
      f4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const v4u kb = *reinterpret_cast<const v4u*>(tile + m * kTilePitch + (quarter * 4 + j) * 16);
        acc = mfma16<DT>(qa[j], kb, acc);
      }
      // lanes 0-15 hold queries 0-3, lanes 16-31 queries 4-7 (rows >= G are zero padding)
      float s = acc[0];
#pragma unroll
      for (int i = 1; i < 4; ++i)
        if (quarter * 4 + i < G) s = fmaxf(s, acc[i]);
      if (G > 4) {
        const float t = __shfl_down(s, 16);  // lane 16+m -> lane m
        s = fmaxf(s, t);
      }
      const int r = wrow + (t0 + u) * 16 + m;
      const u32 key = token_key(s, row0 + r, N, n_sink, n_recent);
      if (quarter == 0) {
        if (HIST)
          s_keys[r] = key;
        else
          kout[r] = key;
      }
    }
  }
  if (HIST) score_hist_epilogue(s_keys, s_hist, keys + (size_t)p * n_pad, hist + (size_t)p * 3 * kBins, row0, N);
}

// Vector-ALU form.  A 16-lane DPP row takes one key row (16 bytes per lane), four rows per
// wave-wide load, fully coalesced; each lane forms G partial dot products with v_dot2 and the
// row sums them through DPP.  Row group r of the wave handles rows 4r..4r+3 of each 16-key tile.
template <int DT, int G, int ROWS, bool HIST>
__global__ __launch_bounds__(256) void qsac_score_valu_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint8_t* __restrict__ reuse_flags,
    u32* __restrict__ keys, u32* __restrict__ hist, int Hq, int Hkv, int64_t N, int64_t n_pad, int n_sink,
    int n_recent) {
  const int p = blockIdx.y;
  if (reuse_flags[p]) return;
  __shared__ u32 s_hist[HIST ? kBins : 1];
  __shared__ __attribute__((aligned(16))) u32 s_keys[HIST ? ROWS : 4];
  if (HIST)
    for (int i = threadIdx.x; i < kBins; i += 256) s_hist[i] = 0;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, r = lane >> 4;
  const int b = p / Hkv, h = p % Hkv;
  const v4u* qg = reinterpret_cast<const v4u*>(q + ((size_t)b * Hq + (size_t)h * G) * kD);
  v4u qf[G];
#pragma unroll
  for (int g = 0; g < G; ++g) qf[g] = qg[g * kRowU4 + c];

  const int64_t row0 = (int64_t)blockIdx.x * ROWS;
  const v4u* Kp = reinterpret_cast<const v4u*>(K + (size_t)p * (size_t)N * kD);
  constexpr int WROWS = ROWS / 4;
  const int wrow = wave * WROWS;
  u32* kout = keys + (size_t)p * n_pad + row0;
  const int64_t last = N - 1;

  for (int t0 = 0; t0 < WROWS / 16; t0 += 2) {
    v4u kv[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        int64_t n = row0 + wrow + (t0 + t) * 16 + r * 4 + u;
        n = n < last ? n : last;
        kv[t][u] = __builtin_nontemporal_load(Kp + n * kRowU4 + c);
      }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      u32 out[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float best = row16_sum(dot8<DT>(qf[0], kv[t][u]));
#pragma unroll
        for (int g = 1; g < G; ++g) best = fmaxf(best, row16_sum(dot8<DT>(qf[g], kv[t][u])));
        const int rr = wrow + (t0 + t) * 16 + r * 4 + u;
        out[u] = token_key(best, row0 + rr, N, n_sink, n_recent);
      }
      if (c == 0) {
        u32* dst = (HIST ? s_keys : kout) + wrow + (t0 + t) * 16 + r * 4;
        *reinterpret_cast<v4u*>(dst) = v4u{out[0], out[1], out[2], out[3]};
      }
    }
  }
  if (HIST) score_hist_epilogue(s_keys, s_hist, keys + (size_t)p * n_pad, hist + (size_t)p * 3 * kBins, row0, N);
}

// ---------------------------------------------------------------- radix select

// LEVEL 1: histogram bits 20..10 of the keys whose bits 31..21 equal the level-0 threshold bin.
// LEVEL 2: histogram bits 9..0 of the keys whose bits 31..10 equal the two-level prefix.
// Every workgroup derives the threshold bin of the level above from that level's finished
// histogram (2048 counters, read from L2) instead of waiting for a separate one-workgroup
// kernel; the first workgroup of a pair leaves it in sel (kSelStride ints per pair: r, bin 0,
// rest after bin 0, bin 1, rest after bin 1) for the kernels that follow.
constexpr int kSelStride = 8;
template <int LEVEL>
__global__ __launch_bounds__(256) void qsac_refine_kernel(const uint8_t* __restrict__ reuse_flags,
                                                          const u32* __restrict__ keys, u32* __restrict__ hist,
                                                          int* __restrict__ sel, int64_t N, int64_t n_pad, int k) {
  const int p = blockIdx.y;
  if (reuse_flags[p]) return;
  __shared__ u32 s_hist[kBins];
  __shared__ int s_wave[5];
  __shared__ int s_res[2];
  u32* hp = hist + (size_t)p * 3 * kBins;
  int* sp = sel + (size_t)p * kSelStride;
  // this workgroup's keys are requested first, so that they travel while the bin of the level above is found
  const int64_t base = (int64_t)blockIdx.x * kSelChunk;
  const v4u* kp = reinterpret_cast<const v4u*>(keys + (size_t)p * n_pad + base);
  v4u kreg[kSelChunk / 4 / 256];
#pragma unroll
  for (int i = 0; i < kSelChunk / 4 / 256; ++i) kreg[i] = kp[i * 256 + threadIdx.x];
  for (int i = threadIdx.x; i < kBins; i += 256) s_hist[i] = 0;
  int above;
  int need = k;
  u32 prefix;
  int shift = 21;
  if (LEVEL == 1) {
    prefix = (u32)find_bin<256>(hp, kBins, need, &above, s_wave, s_res);
    need -= above;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      sp[1] = (int)prefix;
      sp[2] = need;
    }
  } else {
    prefix = (u32)sp[1];
    need = sp[2];
    u32 b1 = (u32)find_bin<256>(hp + kBins, kBins, need, &above, s_wave, s_res);
    need -= above;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      sp[3] = (int)b1;
      sp[4] = need;
    }
    prefix = (prefix << 11) | b1;
    shift = 10;
  }
  const u32 mask = (LEVEL == 1) ? 0x7ffu : 0x3ffu;
  const int sub = (LEVEL == 1) ? 10 : 0;
#pragma unroll
  for (int i = 0; i < kSelChunk / 4 / 256; ++i) {
    const int v = i * 256 + threadIdx.x;
    const v4u kk = kreg[i];
    const int64_t n = base + (int64_t)v * 4;
    if (n + 0 < N && (kk.x >> shift) == prefix) atomicAdd(&s_hist[(kk.x >> sub) & mask], 1u);
    if (n + 1 < N && (kk.y >> shift) == prefix) atomicAdd(&s_hist[(kk.y >> sub) & mask], 1u);
    if (n + 2 < N && (kk.z >> shift) == prefix) atomicAdd(&s_hist[(kk.z >> sub) & mask], 1u);
    if (n + 3 < N && (kk.w >> shift) == prefix) atomicAdd(&s_hist[(kk.w >> sub) & mask], 1u);
  }
  __syncthreads();
  u32* out = hp + LEVEL * kBins;
  for (int bin = threadIdx.x; bin < kBins; bin += 256) {
    u32 c = s_hist[bin];
    if (c) atomicAdd(&out[bin], c);
  }
}

// With the k-th largest key T known exactly: bitmap of keys > T, bitmap of keys == T (64 keys
// per wave-wide ballot), and either a cleared bitmap for the cached tokens (for qsac_diff_kernel)
// or the chunk's two bit counts (chunk_cnt given: for qsac_emit_kernel).
__global__ __launch_bounds__(256) void qsac_mark_kernel(const uint8_t* __restrict__ reuse_flags,
                                                        const u32* __restrict__ keys, const u32* __restrict__ hist,
                                                        u32* __restrict__ bm_new, u32* __restrict__ bm_eq,
                                                        u32* __restrict__ bm_old, int* __restrict__ sel,
                                                        int* __restrict__ chunk_cnt, int64_t N, int64_t n_pad,
                                                        int words, int k) {
  const int p = blockIdx.y;
  if (reuse_flags[p]) return;
  __shared__ int s_wave[5];
  __shared__ int s_res[2];
  __shared__ int s_cnt[2];
  if (threadIdx.x < 2) s_cnt[threadIdx.x] = 0;  // find_bin's barriers come before its use
  const u32* hp = hist + (size_t)p * 3 * kBins;
  int* sp = sel + (size_t)p * kSelStride;
  // this workgroup's keys are requested first, so that they travel while T is put together
  const int64_t base = (int64_t)blockIdx.x * kSelChunk;
  const u32* kp = keys + (size_t)p * n_pad;
  u32 kreg[kSelChunk / 256];
#pragma unroll
  for (int i = 0; i < kSelChunk / 256; ++i) kreg[i] = kp[base + (int64_t)i * 256 + threadIdx.x];
  const u32 b0 = (u32)sp[1], b1 = (u32)sp[3];
  int above, need = sp[4];
  u32 b2 = (u32)find_bin<256>(hp + 2 * kBins, 1024, need, &above, s_wave, s_res);
  need -= above;  // number of keys equal to T that belong to the set (>= 1)
  const u32 T = (b0 << 21) | (b1 << 10) | b2;
  if (blockIdx.x == 0 && threadIdx.x == 0) sp[0] = need;

  const int lane = threadIdx.x & 63;
  u32* gt = bm_new + (size_t)p * words;
  u32* eq = bm_eq + (size_t)p * words;
  u32* old = bm_old + (size_t)p * words;
  const bool clear_old = chunk_cnt == nullptr;
  int cg = 0, ce = 0;  // lane 0: bits of this wave
#pragma unroll
  for (int i = 0; i < kSelChunk / 256; ++i) {
    const int64_t n = base + (int64_t)i * 256 + threadIdx.x;
    const u32 key = kreg[i];
    const bool in = n < N;
    const u64 mg = __ballot(in && key > T);
    const u64 me = __ballot(in && key == T);
    cg += __popcll(mg);
    ce += __popcll(me);
    const int64_t w = n >> 5;  // lane 0 -> low word, lane 32 -> high word of this wave's 64 keys
    if (lane == 0) {
      gt[w] = (u32)mg;
      eq[w] = (u32)me;
      if (clear_old) old[w] = 0;
    } else if (lane == 32) {
      gt[w] = (u32)(mg >> 32);
      eq[w] = (u32)(me >> 32);
      if (clear_old) old[w] = 0;
    }
  }
  if (!clear_old) {
    if (lane == 0) {
      atomicAdd(&s_cnt[0], cg);
      atomicAdd(&s_cnt[1], ce);
    }
    __syncthreads();
    if (threadIdx.x < 2) chunk_cnt[((size_t)p * gridDim.x + blockIdx.x) * 2 + threadIdx.x] = s_cnt[threadIdx.x];
  }
}

// Long contexts (more bitmap words than one workgroup reads quickly): the selected set as an
// ascending token list, written by the whole grid.  Workgroup (chunk, pair) of 256 threads, one
// bitmap word each: the chunks' bit counts (qsac_mark_kernel) give the number of selected tokens
// before the chunk; of the keys equal to the k-th key, the r with the lowest indices overall
// are selected, i.e. those whose rank among the equal keys is below r.  The list goes to
// set_sorted and topk_idx.
__global__ __launch_bounds__(256) void qsac_emit_kernel(const uint8_t* __restrict__ reuse_flags,
                                                        const u32* __restrict__ bm_new,
                                                        const u32* __restrict__ bm_eq,
                                                        const int* __restrict__ chunk_cnt,
                                                        const int* __restrict__ sel, int* __restrict__ set_sorted,
                                                        int* __restrict__ topk_idx, int words, int k, int k_max) {
  const int p = blockIdx.y, c = blockIdx.x, n_chunks = gridDim.x;
  if (reuse_flags[p]) return;
  __shared__ int s_wave[5];
  const int tid = threadIdx.x;
  const int r = sel[(size_t)p * kSelStride];
  const int* cnt = chunk_cnt + (size_t)p * n_chunks * 2;
  // bits of the chunks before this one
  int g_before = 0, e_before = 0;
  for (int cc = tid; cc < c; cc += 256) {
    g_before += cnt[2 * cc];
    e_before += cnt[2 * cc + 1];
  }
  int total;
  (void)block_exclusive_scan<4>(g_before, s_wave, &total);
  g_before = total;
  (void)block_exclusive_scan<4>(e_before, s_wave, &total);
  e_before = total;
  const int w = c * (kSelChunk / 32) + tid;  // words is a multiple of kSelChunk / 32
  u32 bits = bm_new[(size_t)p * words + w];
  if (cnt[2 * c + 1] > 0) {  // uniform: keys equal to the k-th key in this chunk
    u32 e = bm_eq[(size_t)p * words + w];
    const int ce = __popc(e);
    const int rank = e_before + block_exclusive_scan<4>(ce, s_wave, &total);  // equal keys at lower indices
    if (ce && rank + ce > r) {  // keep only the lowest (r - rank) bits of e
      int keep = r - rank;
      u32 kept = 0;
      while (keep > 0 && e) {
        const u32 low = e & (0u - e);
        kept |= low;
        e ^= low;
        --keep;
      }
      e = kept;
    }
    bits |= e;
  }
  int pos = g_before + min(r, e_before) + block_exclusive_scan<4>(__popc(bits), s_wave, &total);
  int* ss = set_sorted + (size_t)p * k_max;
  int* tk = topk_idx + (size_t)p * k;
  while (bits) {
    const int bit = __ffs(bits) - 1;
    bits &= bits - 1;
    if (pos < k) {  // the set has exactly k members; the guard only protects the buffers
      ss[pos] = w * 32 + bit;
      tk[pos] = w * 32 + bit;
    }
    ++pos;
  }
}

// The diff for qsac_emit_kernel's list (k <= kDiffListMax): one workgroup of 1024 threads per
// missing pair, with everything a lookup touches in LDS:
//  1. the ascending list of the set into LDS (l_new);
//  2. every cached token (slot_idx) is looked up in l_new by binary search: found marks the list
//     entry as a hit, not found marks the slot for eviction;
//  3. hit mask, ascending list of tokens to fetch (entries that are no hit), ascending list of
//     evicted slots;
//  4. the i-th evicted slot takes the i-th token to fetch.
// Dynamic LDS: l_new, l_mt, l_ms (k ints each), l_hit (k bytes).
constexpr int kDiffListMax = 8192;
__global__ __launch_bounds__(kDiffThreads) void qsac_diff_list_kernel(
    const uint8_t* __restrict__ reuse_flags, u32* __restrict__ valid, int* __restrict__ slot_idx,
    const int* __restrict__ set_sorted, int* __restrict__ topk_idx, uint8_t* __restrict__ hit_mask,
    int* __restrict__ miss_count, int* __restrict__ miss_slot, int* __restrict__ miss_tok,
    int* __restrict__ fetch_tok, u64* __restrict__ stats, FillSrc src, int Hkv, int k, int k_max) {
  const int p = blockIdx.x;
  if (reuse_flags[p]) {
    report_cached_set(set_sorted, topk_idx, hit_mask, p, k, k_max);
    return;
  }
  constexpr int NT = kDiffThreads;
  constexpr int kMaxSpt = kDiffListMax / NT;
  extern __shared__ int s_lists[];
  __shared__ int s_wave[32];
  int* l_new = s_lists;
  int* l_mt = l_new + k;
  int* l_ms = l_mt + k;
  uint8_t* l_hit = reinterpret_cast<uint8_t*>(l_ms + k);
  const int tid = threadIdx.x;
  int* sl = slot_idx + (size_t)p * k_max;
  const int* ss = set_sorted + (size_t)p * k_max;
  uint8_t* hm = hit_mask + (size_t)p * k;
  int* ms = miss_slot + (size_t)p * k_max;
  int* mt = miss_tok + (size_t)p * k_max;
  int* ft = fetch_tok + (size_t)p * k_max;
  const bool was_valid = valid[p] != 0;
  // the thread's slots (and, in 3, its entries of the list): [j0, j1), at most kMaxSpt
  const int spt = (k + NT - 1) / NT;
  const int j0 = min(tid * spt, k), j1 = min(j0 + spt, k);
  int mytok[kMaxSpt];
#pragma unroll
  for (int i = 0; i < kMaxSpt; ++i) mytok[i] = (was_valid && j0 + i < j1) ? sl[j0 + i] : -1;
  // 1
  for (int j = tid; j < k; j += NT) {
    l_new[j] = ss[j];
    l_hit[j] = 0;
    ft[j] = -1;  // slots that keep their row; 4 names the others
  }
  __syncthreads();
  // 2: all lookups of a thread advance together, one probe each per round, without branches:
  // pos = number of list entries below the token
  int pos[kMaxSpt];
#pragma unroll
  for (int i = 0; i < kMaxSpt; ++i) pos[i] = 0;
  int top = 1;
  while (top < k) top <<= 1;
  for (int step = top; step > 0; step >>= 1) {
#pragma unroll
    for (int i = 0; i < kMaxSpt; ++i) {
      if (i < spt) {  // uniform: the probes are bound by the LDS, so none is spent on slots nobody has
        const int nxt = pos[i] + step;
        const int probe = l_new[min(nxt, k) - 1];
        pos[i] = (nxt <= k && probe < mytok[i]) ? nxt : pos[i];
      }
    }
  }
  bool evict[kMaxSpt];
  int ce = 0;
#pragma unroll
  for (int i = 0; i < kMaxSpt; ++i) {
    evict[i] = false;
    if (j0 + i < j1) {
      const bool found = was_valid && pos[i] < k && l_new[pos[i]] == mytok[i];
      if (found) l_hit[pos[i]] = 1;  // slots hold distinct tokens: one writer per entry
      evict[i] = !found;
      ce += !found;
    }
  }
  int total;
  int je = block_exclusive_scan<NT / 64>(ce, s_wave, &total);  // its barriers also publish l_hit
  const int m = total;
#pragma unroll
  for (int i = 0; i < kMaxSpt; ++i)
    if (evict[i]) {
      l_ms[je] = j0 + i;
      ms[je] = j0 + i;
      ++je;
    }
  // 3
  int cm = 0;
#pragma unroll
  for (int i = 0; i < kMaxSpt; ++i)
    if (j0 + i < j1) cm += !l_hit[j0 + i];
  int jm = block_exclusive_scan<NT / 64>(cm, s_wave, &total);
#pragma unroll
  for (int i = 0; i < kMaxSpt; ++i)
    if (j0 + i < j1) {
      const bool hit = l_hit[j0 + i] != 0;
      hm[j0 + i] = (uint8_t)hit;
      if (!hit) {
        if (jm < k) {
          l_mt[jm] = l_new[j0 + i];
          mt[jm] = l_new[j0 + i];
        }
        ++jm;
      }
    }
  __syncthreads();
  // 4
  for (int i = tid; i < m; i += NT) {
    const int slot = l_ms[i], tok = l_mt[i];
    sl[slot] = tok;
    ft[slot] = tok;
  }
  if (tid == 0) {
    miss_count[p] = m;
    valid[p] = 1;
    atomicAdd(&stats[3], (u64)(k - m));
    atomicAdd(&stats[4], (u64)m);
    if (src.slot[p % Hkv] >= 0)
      atomicAdd(&stats[5], (u64)m);
    else if (src.host_row_bytes)
      atomicAdd(&stats[7], (u64)m * (u64)src.host_row_bytes);
  }
}

// ---------------------------------------------------------------- diff

// Shared by the one-workgroup select (bitmaps in LDS) and the large-N diff kernel (bitmaps in
// the workspace).  Thread t of NT owns a contiguous run of bitmap words.  nw holds the keys above
// the k-th key on entry and the selected set on exit.
//  A. ties: of the keys equal to the k-th key, the r with the lowest indices join the set;
//     (the bitmaps are walked wave by wave, 64 coalesced words at a time, ranks by DPP scans;
//     WPL bounds the words a lane holds: words <= 64 * WPL * NT / 64)
//  B. bitmap of the tokens cached before the step (from slot_idx);
//  C. ascending index list, hit mask, ascending list of tokens to fetch;
//  D. ascending list of slots whose token left the set (its counts travel with C's through one exchange);
//  E. the i-th such slot takes the i-th token to fetch (slot table and fetch_tok).
// STAGE: the caller gives room in LDS (DiffStage: k ints each for ms, mt and tk, k bytes for hm).  The four
// lists are built there and leave with coalesced stores, and E takes the miss lists from there (scattered 4-byte
// stores from every lane are what the emission otherwise waits on).
// skip_ties: the caller has already put every key equal to the k-th key into nw (r and eq are not read).
struct DiffStage {
  int* ms = nullptr;
  int* mt = nullptr;
  int* tk = nullptr;
  uint8_t* hm = nullptr;
};

// The slot tokens diff_phases keeps in registers (thread t: slots [t * spt, t * spt + spt) with spt = ceil(k / NT),
// if spt <= 4), for callers that can request them long before the diff starts.  Reads the slot table whether or
// not the cache is valid (the table exists either way; B and D ignore what an invalid cache held).
template <int NT>
__device__ __forceinline__ void diff_slot_tokens(const int* __restrict__ sl, int k, int tok[4]) {
  const int spt = (k + NT - 1) / NT;
  const int j0 = min((int)threadIdx.x * spt, k), j1 = min(j0 + spt, k);
#pragma unroll
  for (int i = 0; i < 4; ++i) tok[i] = (spt <= 4 && j0 + i < j1) ? sl[j0 + i] : 0;
}

template <int NT, int WPL, bool STAGE = false>
__device__ __forceinline__ void diff_phases(u32* __restrict__ nw, const u32* __restrict__ eq,
                                            u32* __restrict__ old, bool was_valid, int r, int words,
                                            int k, int* __restrict__ sl, int* __restrict__ ss,
                                            int* __restrict__ tk, uint8_t* __restrict__ hm, int* __restrict__ ms,
                                            int* __restrict__ mt, int* __restrict__ ft,
                                            int* __restrict__ miss_count_p, u32* __restrict__ valid_p,
                                            u64* __restrict__ stats, bool resident, int host_row_bytes,
                                            int* s_wave /*[3 * NT / 64]*/, DiffStage st = DiffStage(),
                                            bool skip_ties = false, const int* pre_tok = nullptr) {
  constexpr int NW = NT / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // Wave w owns the contiguous words [wb, we); lane l takes words wb + l, wb + l + 64, ... (at most
  // WPL of them), so that every bitmap read is coalesced and index order is (round, lane).  A lane
  // keeps its words in registers: each bitmap is read from memory once, in one round trip.
  const int wpw = ((words + NW - 1) / NW + 63) & ~63;
  const int wb = min(wave * wpw, words), we = min(wb + wpw, words);
  const int rounds = wpw >> 6;  // <= WPL, uniform over the workgroup
  // thread t owns the contiguous slots [j0, j1); up to four of their tokens are requested now and
  // kept in registers for B and D (with more slots per thread they are re-read where needed)
  const int spt = (k + NT - 1) / NT;
  const int j0 = min(tid * spt, k), j1 = min(j0 + spt, k);
  const bool slots_in_regs = spt <= 4;  // uniform
  int mytok[4] = {0, 0, 0, 0};
  if (pre_tok) {  // the caller has read them already (diff_slot_tokens)
#pragma unroll
    for (int i = 0; i < 4; ++i) mytok[i] = pre_tok[i];
  } else if (was_valid && slots_in_regs) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (j0 + i < j1) mytok[i] = sl[j0 + i];
  }
  for (int j = tid; j < k; j += NT) ft[j] = -1;  // slots that keep their row; E names the others
  // A
  if (!skip_ties) {
    u32 ev[WPL];
    int ceq = 0;
#pragma unroll
    for (int u = 0; u < WPL; ++u) {
      const int w = wb + u * 64 + lane;
      ev[u] = (u < rounds && w < we) ? eq[w] : 0u;
      ceq += __popc(ev[u]);
    }
    ceq = __builtin_amdgcn_readlane(wave_inclusive_scan(ceq), 63);
    int total;
    int run = wave_totals_exclusive<NW>(ceq, s_wave, &total);
    if (total == r) {  // every key equal to the k-th key belongs to the set (the usual case: it is alone)
#pragma unroll
      for (int u = 0; u < WPL; ++u)
        if (ev[u]) nw[wb + u * 64 + lane] |= ev[u];
    } else {
#pragma unroll
      for (int u = 0; u < WPL; ++u) {
        if (u < rounds) {  // uniform: every lane takes part in the scan
          u32 e = ev[u];
          const int c = __popc(e);
          const int inc = wave_inclusive_scan(c);
          const int rank = run + inc - c;  // keys equal to the k-th key at lower indices
          if (c && rank + c > r) {         // keep only the lowest (r - rank) bits of e
            int keep = r - rank;
            u32 kept = 0;
            while (keep > 0 && e) {
              u32 low = e & (0u - e);
              kept |= low;
              e ^= low;
              --keep;
            }
            e = kept;
          }
          if (e) nw[wb + u * 64 + lane] |= e;
          run += __builtin_amdgcn_readlane(inc, 63);
        }
      }
    }
  }
  // B
  if (was_valid) {
    if (slots_in_regs) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (j0 + i < j1) atomicOr(&old[mytok[i] >> 5], 1u << (mytok[i] & 31));
    } else {
      for (int j = j0; j < j1; ++j) {
        const int tok = sl[j];
        atomicOr(&old[tok >> 5], 1u << (tok & 31));
      }
    }
  }
  __syncthreads();
  // C and D share one exchange of wave totals
  u32 av[WPL], ov[WPL];
  int cn = 0, cm = 0;
#pragma unroll
  for (int u = 0; u < WPL; ++u) {
    const int w = wb + u * 64 + lane;
    const bool in = u < rounds && w < we;
    av[u] = in ? nw[w] : 0u;
    ov[u] = in ? old[w] : 0u;
    cn += __popc(av[u]);
    cm += __popc(av[u] & ~ov[u]);
  }
  // D, counting: this thread's slots whose token left the set (all of them if the cache was invalid)
  bool evict[4] = {false, false, false, false};
  int ce = 0;
  if (slots_in_regs) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (j0 + i < j1) {
        evict[i] = !was_valid || !((nw[mytok[i] >> 5] >> (mytok[i] & 31)) & 1u);
        ce += evict[i];
      }
  } else {
    for (int j = j0; j < j1; ++j) {
      bool e = true;
      if (was_valid) {
        const int tok = sl[j];
        e = !((nw[tok >> 5] >> (tok & 31)) & 1u);
      }
      ce += e;
    }
  }
  cn = __builtin_amdgcn_readlane(wave_inclusive_scan(cn), 63);
  cm = __builtin_amdgcn_readlane(wave_inclusive_scan(cm), 63);
  const int inc_e = wave_inclusive_scan(ce);
  int runn, runm, rune, m;
  wave_totals_exclusive3<NW, false>(cn, cm, __builtin_amdgcn_readlane(inc_e, 63), s_wave, &runn, &runm, &rune, &m);
  // C, emission
#pragma unroll
  for (int u = 0; u < WPL; ++u) {
    if (u < rounds) {
      u32 a = av[u];
      const u32 o = ov[u];
      const int c1 = __popc(a), c2 = __popc(a & ~o);
      const int i1 = wave_inclusive_scan(c1), i2 = wave_inclusive_scan(c2);
      int jn = runn + i1 - c1, jm = runm + i2 - c2;
      const int w = wb + u * 64 + lane;
      while (a) {
        const int bit = __ffs(a) - 1;
        a &= a - 1;
        const int tok = w * 32 + bit;
        const bool hit = (o >> bit) & 1u;
        if (jn < k) {  // the set has exactly k members; the guard only protects the buffers
          if (STAGE) {
            st.tk[jn] = tok;
            st.hm[jn] = (uint8_t)hit;
          } else {
            tk[jn] = tok;
            ss[jn] = tok;
            hm[jn] = (uint8_t)hit;
          }
        }
        ++jn;
        if (!hit) {
          if (jm < k) (STAGE ? st.mt : mt)[jm] = tok;
          ++jm;
        }
      }
      runn += __builtin_amdgcn_readlane(i1, 63);
      runm += __builtin_amdgcn_readlane(i2, 63);
    }
  }
  // D, emission
  int je = rune + inc_e - ce;
  if (slots_in_regs) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (evict[i]) {
        (STAGE ? st.ms : ms)[je] = j0 + i;
        ++je;
      }
  } else {
    for (int j = j0; j < j1; ++j) {
      bool e = true;
      if (was_valid) {
        const int tok = sl[j];
        e = !((nw[tok >> 5] >> (tok & 31)) & 1u);
      }
      if (e) {
        (STAGE ? st.ms : ms)[je] = j;
        ++je;
      }
    }
  }
  __syncthreads();
  if (STAGE) {
    for (int i = tid; i < k; i += NT) {
      const int tok = st.tk[i];
      tk[i] = tok;
      ss[i] = tok;
      hm[i] = st.hm[i];
    }
  }
  // E
  for (int i = tid; i < m; i += NT) {
    const int slot = (STAGE ? st.ms : ms)[i], tok = (STAGE ? st.mt : mt)[i];
    sl[slot] = tok;
    ft[slot] = tok;
    if (STAGE) {
      ms[i] = slot;
      mt[i] = tok;
    }
  }
  if (tid == 0) {
    *miss_count_p = m;
    *valid_p = 1;
    atomicAdd(&stats[3], (u64)(k - m));
    atomicAdd(&stats[4], (u64)m);
    if (resident)
      atomicAdd(&stats[5], (u64)m);
    else if (host_row_bytes)
      atomicAdd(&stats[7], (u64)m * (u64)host_row_bytes);
  }
}

// Large-N path: one workgroup per missing pair, bitmaps in the workspace (made by qsac_mark_kernel).
// WPL: bitmap words a lane holds; words <= 1024 * WPL.
template <int WPL>
__global__ __launch_bounds__(kDiffThreads) void qsac_diff_kernel(
    const uint8_t* __restrict__ reuse_flags, u32* __restrict__ valid, u32* __restrict__ bm_new,
    const u32* __restrict__ bm_eq, u32* __restrict__ bm_old, const int* __restrict__ sel_r,
    int* __restrict__ slot_idx, int* __restrict__ set_sorted, int* __restrict__ topk_idx,
    uint8_t* __restrict__ hit_mask, int* __restrict__ miss_count, int* __restrict__ miss_slot,
    int* __restrict__ miss_tok, int* __restrict__ fetch_tok, u64* __restrict__ stats, FillSrc src, int Hkv,
    int words, int k, int k_max) {
  const int p = blockIdx.x;
  if (reuse_flags[p]) {
    report_cached_set(set_sorted, topk_idx, hit_mask, p, k, k_max);
    return;
  }
  __shared__ int s_wave[64];
  diff_phases<kDiffThreads, WPL>(bm_new + (size_t)p * words, bm_eq + (size_t)p * words, bm_old + (size_t)p * words,
                            valid[p] != 0, sel_r[(size_t)p * kSelStride], words, k, slot_idx + (size_t)p * k_max,
                            set_sorted + (size_t)p * k_max, topk_idx + (size_t)p * k, hit_mask + (size_t)p * k,
                            miss_slot + (size_t)p * k_max, miss_tok + (size_t)p * k_max,
                            fetch_tok + (size_t)p * k_max, miss_count + p, valid + p, stats,
                            src.slot[p % Hkv] >= 0, src.host_row_bytes, s_wave);
}

// OR over aligned groups of 8 lanes (DPP: xor 1, xor 2, then mirror within each half row).
__device__ __forceinline__ u32 or8(u32 v) {
  v |= (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);
  v |= (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true);
  v |= (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, true);
  return v;
}

struct SelArgs {
  const uint8_t* reuse_flags;
  const u32* keys;
  u32* valid;
  int* slot_idx;
  int* set_sorted;
  int* topk_idx;
  uint8_t* hit_mask;
  int* miss_count;
  int* miss_slot;
  int* miss_tok;
  int* fetch_tok;
  u64* stats;
  int64_t N, n_pad;
  int Hkv, k, k_max, bm_words, list_cap, r_sample;
};

// Small-N path (N <= kSmallMaxN): one workgroup of NT threads per missing pair selects and diffs
// in one go.  Thread t keeps key vectors t, t + NT, ... (VPT of them, 4 keys each) in registers,
// so the keys are read from memory once.
//
// Full path: three histogram passes over all keys (11 + 11 + 10 bits) pin the k-th largest key
// T exactly; a fourth pass turns "key > T" and "key == T" into LDS bitmaps.
//
// Guided path (r_sample > 0): a histogram of the top 12 key bits of 4 keys per thread (a 1/VPT
// sample, spread over the context) gives a bound g, the lower edge of the bin that holds the
// sample's r_sample-th largest key.  r_sample is chosen so that the number of keys >= g falls
// between k and list_cap with near certainty.  k <= #{key >= g} proves T >= g, i.e. every key of
// the top-k, and every key equal to T, is among those candidates: they are compacted into an
// LDS list (each wave appends to its own part of the list, by ballot rank, and stays its only
// reader) and T is pinned over the list only: one histogram of d = key - g in bins 2^kCandShift
// wide (the candidates share their leading key bits, so digits of the key itself would pile them
// into a handful of bins) names the bin that holds T, and the few keys of that bin are ranked
// directly (each wave by itself, one key per lane).  The full path runs instead if fewer than k
// keys reach g or a wave's part of the list overflows; the three plain levels run over the list
// if T's bin holds more than 64 keys or T lies too far above g for the bins.  The result is the
// same every way.  When every key equal to T belongs to the set (nearly always: T is alone) the
// bitmap pass puts them into the set directly and the diff skips its tie phase.
//
// Dynamic LDS (s_dyn): three bitmaps of bm_words words, then list_cap (key, index) entries of 8 bytes (the diff's
// staging lists take that room over once T is known).
template <int VPT, int NT>
__device__ __forceinline__ void select_small_body(const SelArgs& A, const FillSrc& src, int p, u32* s_dyn) {
  constexpr int NV = VPT;
  __shared__ __align__(16) u32 s_hist[kHistCopies * kHistPitch];
  __shared__ int s_wave[64];
  __shared__ int s_res[3];
  __shared__ u32 s_small[64];
  __shared__ int s_flag[2];  // [0] a wave ran out of list room, [1] keys gathered in s_small
  constexpr int NW = NT / 64;
  const int bm_words = A.bm_words, k = A.k, k_max = A.k_max;
  u32* s_new = s_dyn;
  u32* s_eq = s_dyn + bm_words;
  u32* s_old = s_dyn + 2 * bm_words;
  u64* l_ent = reinterpret_cast<u64*>(s_dyn + 3 * bm_words);  // bm_words is even: 8-byte aligned
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool reused = A.reuse_flags[p] != 0;
  const v4u* kp4 = reinterpret_cast<const v4u*>(A.keys + (size_t)p * A.n_pad);
  const int n = (int)A.N;
  const int nvec = (n + 3) >> 2;  // n_pad is a multiple of 8192, so whole vectors can be read
  const int words = (n + 31) >> 5;

  // Keys at and past N read as 0 (the scoring kernel writes 0 there, vectors past the end are
  // zeroed here).  0 is below the key of every finite score, so it never reaches the k-th key's
  // bin, never matches a prefix and never compares above or equal to T or a bound: no range
  // checks below.
  v4u kreg[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int v = tid + i * NT;
    kreg[i] = v < nvec ? kp4[v] : v4u{0, 0, 0, 0};
  }
  // requested now, used by the diff at the end
  const bool was_valid = A.valid[p] != 0;
  int pre_tok[4];
  diff_slot_tokens<NT>(A.slot_idx + (size_t)p * k_max, k, pre_tok);
  // The gate's verdict is looked at only now, with the key loads already on their way: a pair that missed does
  // not wait for the flag and then again for its keys (a pair that reused drops the loads it never needed).
  if (reused) {
    report_cached_set(A.set_sorted, A.topk_idx, A.hit_mask, p, k, k_max);
    return;
  }
  lds_zero<NT>(s_dyn, 3 * bm_words);  // the three bitmaps are adjacent

  int need = k, above;
  u32 prefix = 0;
  // level 0: bits 31..21; level 1: bits 20..10 under the level-0 bin; level 2: bits 9..0
  auto level_shift = [](int level) { return level == 1 ? 21 : 10; };  // from level 1 on, key >> shift == prefix
  auto level_sub = [](int level) { return level == 0 ? 21 : (level == 1 ? 10 : 0); };
  auto level_mask = [](int level) { return level == 2 ? 0x3ffu : 0x7ffu; };

  bool guided = false;    // uniform over the workgroup
  bool all_ties = false;  // uniform: every key equal to the k-th key belongs to the set and is already in s_new
  u32 bound = 0;
  if (A.r_sample > 0) {
    // the sample's 4096 bins, and behind them the kCandBins bins of the candidates' first level
    lds_zero<NT>(s_hist, 4096 + kCandBins);
    if (tid < 2) s_flag[tid] = 0;
    __syncthreads();
    constexpr int S = 4096 / NT;  // sample keys per thread, spread over its vectors
#pragma unroll
    for (int j = 0; j < S; ++j) {
      u32 key;
      if (NV >= S) {
        key = kreg[j * (NV / S)].x;
      } else {
        constexpr int per = S / (NV < S ? NV : S);  // 2 or 4 sample keys per vector
        const v4u& q = kreg[(j / per) % NV];
        const int c = (j % per) * (4 / per);
        key = c == 0 ? q.x : c == 1 ? q.y : c == 2 ? q.z : q.w;
      }
      atomicAdd(&s_hist[key >> 20], 1u);
    }
    __syncthreads();
    bound = (u32)find_bin<NT, 1>(s_hist, 4096, A.r_sample, &above, s_wave, s_res) << 20;
  }
  if (bound != 0u) {
    // Candidates (key >= bound) into the list as (key, index) entries.  The order of the list is irrelevant
    // (histograms and bitmaps do not depend on it): every wave appends to its own part of the list, each key slot
    // by ballot rank, and is the only reader of that part afterwards, so no count has to be exchanged first.  The
    // last entry of a part only catches what does not fit; a wave that gets that far calls the guided path off.
    constexpr int kMine = kSelectListCap / NT;  // a lane's share of its wave's entries
    const int part = min(A.list_cap / NW, 64 * kMine);
    u64* my_ent = l_ent + wave * part;
    int n_mine = 0;  // wave-uniform
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const u32 ks[4] = {kreg[i].x, kreg[i].y, kreg[i].z, kreg[i].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool c = ks[j] >= bound;
        const u64 m = __ballot(c);
        if (c) {
          const int pos = (int)__builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, (u32)n_mine));
          my_ent[min(pos, part - 1)] = ((u64)ks[j] << 32) | (u32)(4 * (tid + i * NT) + j);
        }
        n_mine += __popcll(m);
      }
    }
    if (n_mine > part - 1) {
      n_mine = 0;
      if (lane == 0) s_flag[0] = 1;
    }
    // From here on a lane keeps its share of the wave's entries (lane, lane + 64, ...) in registers.
    u32 ekey[kMine];
    int eidx[kMine];
#pragma unroll
    for (int i = 0; i < kMine; ++i) {
      u64 ent = 0ull;  // key 0: below every bound
      if (i * 64 < n_mine)  // wave-uniform: the rounds past the wave's count cost a scalar branch
        if (i * 64 + lane < n_mine) ent = my_ent[i * 64 + lane];
      ekey[i] = (u32)(ent >> 32);
      eidx[i] = (int)(u32)ent;
    }
    // All candidates share the leading key bits, so the radix digit is taken from d = key - bound: d >> kCandShift
    // in kCandBins bins (the last bin also takes everything further up).  A wave counts its own entries: no
    // barrier since the compaction.
    u32* const hist1 = s_hist + 4096;
#pragma unroll
    for (int i = 0; i < kMine; ++i)
      if (i * 64 < n_mine)
        if (ekey[i] != 0u) atomicAdd(&hist1[min((ekey[i] - bound) >> kCandShift, (u32)kCandBins - 1u)], 1u);
    __syncthreads();
    int in_bin;
    const int b1 = find_bin<NT, 1>(hist1, kCandBins, k, &above, s_wave, s_res, nullptr, &in_bin);
    // b1 >= 0: at least k candidates, which proves that the k-th key is among them
    guided = b1 >= 0 && s_flag[0] == 0;
    if (guided) {
      if (b1 != kCandBins - 1 && in_bin <= 64) {
        // The k-th key is one of the few keys of bin b1: they are gathered and every wave ranks them by itself.
        need -= above;
        const u32 lo = bound + ((u32)b1 << kCandShift);
#pragma unroll
        for (int i = 0; i < kMine; ++i)
          if (i * 64 < n_mine)
            if (ekey[i] - lo < (1u << kCandShift)) s_small[atomicAdd(&s_flag[1], 1)] = ekey[i];
        __syncthreads();
        const int n_small = __builtin_amdgcn_readfirstlane(in_bin);
        const u32 v = lane < n_small ? s_small[lane] : 0u;
        int gt = 0, eq = 0;  // keys of the bin above / equal to this lane's (itself included)
        for (int j = 0; j < n_small; ++j) {
          const u32 x = (u32)__builtin_amdgcn_readlane((int)v, j);
          gt += (int)(x > v);
          eq += (int)(x == v);
        }
        const u64 holds = __ballot(lane < n_small && gt < need && need <= gt + eq);
        const int from = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)holds) - 1);
        prefix = (u32)__builtin_amdgcn_readlane((int)v, from);
        need -= __builtin_amdgcn_readlane(gt, from);
        all_ties = need == __builtin_amdgcn_readlane(eq, from);
      } else {
        // too many keys share that bin, or the k-th key lies further above the bound than the bins resolve: the
        // plain three levels over the list
#pragma unroll
        for (int level = 0; level < 3; ++level) {
          for (int i = tid; i < kBins; i += NT) s_hist[i] = 0;
          __syncthreads();
#pragma unroll
          for (int i = 0; i < kMine; ++i)
            if (ekey[i] != 0u && (level == 0 || (ekey[i] >> level_shift(level)) == prefix))
              atomicAdd(&s_hist[(ekey[i] >> level_sub(level)) & level_mask(level)], 1u);
          __syncthreads();
          const u32 bsel = (u32)find_bin<NT, 1>(s_hist, level == 2 ? 1024 : kBins, need, &above, s_wave, s_res);
          need -= above;
          prefix = level == 0 ? bsel : (prefix << (level == 1 ? 11 : 10)) | bsel;
        }
      }
      const u32 T = prefix;  // >= bound > 0: the empty entries (key 0) fall through
#pragma unroll
      for (int i = 0; i < kMine; ++i) {
        if (i * 64 < n_mine) {
          if (ekey[i] > T || (all_ties && ekey[i] == T))
            atomicOr(&s_new[eidx[i] >> 5], 1u << (eidx[i] & 31));
          else if (ekey[i] == T)
            atomicOr(&s_eq[eidx[i] >> 5], 1u << (eidx[i] & 31));
        }
      }
    }
  }
  if (!guided) {
    u32* my_hist = s_hist + (tid & (kHistCopies - 1)) * kHistPitch;
#pragma unroll
    for (int level = 0; level < 3; ++level) {
      for (int i = tid; i < kHistCopies * kHistPitch; i += NT) s_hist[i] = 0;
      __syncthreads();
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const u32 ks[4] = {kreg[i].x, kreg[i].y, kreg[i].z, kreg[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (level == 0 || (ks[j] >> level_shift(level)) == prefix)
            atomicAdd(&my_hist[(ks[j] >> level_sub(level)) & level_mask(level)], 1u);
      }
      __syncthreads();
      const u32 bsel =
          (u32)find_bin<NT, kHistCopies>(s_hist, level == 2 ? 1024 : kBins, need, &above, s_wave, s_res);
      need -= above;
      prefix = level == 0 ? bsel : (prefix << (level == 1 ? 11 : 10)) | bsel;
    }
    const u32 T = prefix;
    // bitmaps: a key vector is a nibble; 8 neighbouring lanes hold the 8 nibbles of one word
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int v = tid + i * NT;
      const u32 ks[4] = {kreg[i].x, kreg[i].y, kreg[i].z, kreg[i].w};
      u32 g = 0, q = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        g |= (u32)(ks[j] > T) << j;
        q |= (u32)(ks[j] == T) << j;
      }
      const int sh = (v & 7) * 4;
      g = or8(g << sh);
      if (__ballot(q != 0)) q = or8(q << sh);  // uniform over the wave; keys equal to T are rare
      if ((v & 7) == 0 && (v >> 3) < words) {
        s_new[v >> 3] = g;
        s_eq[v >> 3] = q;
      }
    }
  }
  // prefix: the k-th largest key; `need` of the keys equal to it belong to the set
  if (tid == 0 && guided) atomicAdd(&A.stats[6], 1ull);
  __syncthreads();
  // 65536 keys = 2048 bitmap words.  The candidate list is dead by now: its room stages the diff's lists if
  // they fit.
#define QSAC_DIFF_ARGS                                                                                              \
  s_new, s_eq, s_old, was_valid, need, words, k, A.slot_idx + (size_t)p * k_max,                                    \
      A.set_sorted + (size_t)p * k_max, A.topk_idx + (size_t)p * k, A.hit_mask + (size_t)p * k,                      \
      A.miss_slot + (size_t)p * k_max, A.miss_tok + (size_t)p * k_max, A.fetch_tok + (size_t)p * k_max,              \
      A.miss_count + p, A.valid + p, A.stats, src.slot[p % A.Hkv] >= 0, src.host_row_bytes, s_wave
  if (3 * k + (k + 3) / 4 <= 2 * A.list_cap) {
    int* const room = reinterpret_cast<int*>(l_ent);
    DiffStage st;
    st.ms = room;
    st.mt = room + k;
    st.tk = room + 2 * k;
    st.hm = reinterpret_cast<uint8_t*>(room + 3 * k);
    diff_phases<NT, 2048 / NT, true>(QSAC_DIFF_ARGS, st, all_ties, pre_tok);
  } else {
    diff_phases<NT, 2048 / NT, false>(QSAC_DIFF_ARGS, DiffStage(), all_ties, pre_tok);
  }
#undef QSAC_DIFF_ARGS
}

template <int VPT, int NT>
__global__ __launch_bounds__(NT) void qsac_select_small_kernel(SelArgs A, FillSrc src) {
  extern __shared__ __align__(16) u32 s_dyn[];
  select_small_body<VPT, NT>(A, src, blockIdx.x, s_dyn);
}

// Mid-N path (kSmallMaxN < N <= kStreamMaxN): the keys of a pair no longer fit one workgroup's registers, but its
// bitmaps still fit one workgroup's LDS.  The scoring kernel has left the exact level-0 histogram (top 11 key
// bits); its bin b0 of the k-th key T splits the keys into "above b0" (in the set for sure), "below" (out) and the
// bin's own keys, the only undecided ones.
//
// Grid (chunks of 4 * kStreamChunkVec * NT keys, pairs), NT threads.  Every workgroup of a pair derives b0 (same histogram, same
// answer) and appends its chunk's keys at or above the bin to the pair's list in the workspace (`glist`: a wave
// reserves room with one atomic add and fills it by ballot rank; the list's length is known beforehand from the
// histogram).  The workgroup that finishes last (a counter per pair; entries and counter are device-scope atomics) goes on
// alone: entries above the bin go straight into the "selected" bitmap in LDS, T is pinned over the rest by one
// histogram of the bits below the bin's and a direct rank among the few keys of T's fine bin (or one more level
// if they are many), then bitmaps and the diff, as in the small-N path.  Nobody waits for anybody: the other
// workgroups are gone by then.
//
// If the histogram says the list would not hold the keys at or above the bin (heavy ties), workgroup 0 of the pair
// does the job alone, streaming the pair's keys (they were just written and sit in the L2) as often as it takes:
// a histogram pass descends one radix level (11, then 10 bits), and as soon as the bin of T holds few enough keys
// they are compacted into an LDS list (each wave its own part, as in the small-N path) and treated as above; after
// the last level T is known exactly and one more pass turns "key > T" and "key == T" into the bitmaps.
// Same result as the grid-wide kernels, which keep the contexts above kStreamMaxN.
//
// sync: kSelStride ints per pair, [0] list entries reserved, [1] workgroups done; zero between launches (the last
// workgroup leaves them so).  Dynamic LDS (s_dyn): three bitmaps of bm_words words, then list_cap entries of 8 bytes.
constexpr int kStreamMaxN = 131072;   // three bitmaps of N bits, the list and the histogram share the LDS
constexpr int kStreamLimit = 4096;    // undecided keys the compaction into LDS is tried with (half the list)
constexpr int kStreamChunkVec = 8;    // key vectors per thread of a workgroup's chunk (32768 keys with 1024 threads)
constexpr int kStreamListCap = 16384; // entries of a pair's list in the workspace (the last workgroup holds them in registers)

template <int NT>
__global__ __launch_bounds__(NT) void qsac_select_stream_kernel(SelArgs A, const u32* __restrict__ hist,
                                                                u64* __restrict__ glist, int gcap,
                                                                int* __restrict__ sync, FillSrc src) {
  extern __shared__ __align__(16) u32 s_dyn[];
  __shared__ __align__(16) u32 s_hist[kCandBins];
  __shared__ int s_wave[64];
  __shared__ int s_res[3];
  __shared__ u32 s_small[64];
  __shared__ int s_flag[3];  // [0] a wave ran out of list room, [1] keys gathered in s_small, [2] arrival ticket
  constexpr int NW = NT / 64;
  constexpr int kMine = kStreamListCap / NT;  // entries a thread keeps in registers
  constexpr int kBatch = 8;                   // key vectors a thread has in flight when streaming
  const int p = blockIdx.y, chunk = blockIdx.x, n_chunks = gridDim.x;
  const int bm_words = A.bm_words, k = A.k, k_max = A.k_max;
  if (A.reuse_flags[p]) {
    if (chunk == 0) report_cached_set(A.set_sorted, A.topk_idx, A.hit_mask, p, k, k_max);
    return;
  }
  u32* s_new = s_dyn;
  u32* s_eq = s_dyn + bm_words;
  u32* s_old = s_dyn + 2 * bm_words;
  u64* l_ent = reinterpret_cast<u64*>(s_dyn + 3 * bm_words);  // bm_words is even: 8-byte aligned
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const v4u* kp4 = reinterpret_cast<const v4u*>(A.keys + (size_t)p * A.n_pad);
  const int n = (int)A.N;
  const int nvec = (n + 3) >> 2;  // keys past N inside the last vector are 0: below every bin that matters
  const int words = (n + 31) >> 5;

  // this workgroup's chunk of the keys, requested before the histogram is looked at (a workgroup that turns out
  // to have nothing to do drops them)
  v4u q[kStreamChunkVec];
#pragma unroll
  for (int u = 0; u < kStreamChunkVec; ++u) {
    const int v = (chunk * kStreamChunkVec + u) * NT + tid;
    q[u] = v < nvec ? kp4[v] : v4u{0, 0, 0, 0};
  }
  // level 0 comes from the scoring kernel: bits 31..21
  int need = k, above = 0, in_bin = 0;
  u32 prefix = (u32)find_bin<NT, 1>(hist + (size_t)p * 3 * kBins, kBins, need, &above, s_wave, s_res, nullptr, &in_bin);
  need -= above;
  int shift = 21;  // key >> shift == prefix names the bin of T; 0 once T is known exactly
  const int n_list = above + in_bin;  // keys at or above the bin
  const bool shared = n_list <= min(gcap, kStreamListCap);

  u32 ekey[kMine];  // the entries this thread works on (key 0: none)
  int eidx[kMine];
  int my_rounds = 0;  // rounds of ekey / eidx that may hold entries (wave-uniform)
  bool have_list = false;
  bool was_valid = false;
  int pre_tok[4] = {0, 0, 0, 0};

  if (shared) {
    u64* gl = glist + (size_t)p * gcap;
    int* sy = sync + (size_t)p * kSelStride;
    int cnt = 0;
#pragma unroll
    for (int u = 0; u < kStreamChunkVec; ++u)
      cnt += __popcll(__ballot((q[u].x >> 21) >= prefix)) + __popcll(__ballot((q[u].y >> 21) >= prefix)) +
             __popcll(__ballot((q[u].z >> 21) >= prefix)) + __popcll(__ballot((q[u].w >> 21) >= prefix));
    int at = 0;
    if (cnt > 0) {  // wave-uniform
      if (lane == 0) at = __hip_atomic_fetch_add(&sy[0], cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      at = __builtin_amdgcn_readfirstlane(at);
#pragma unroll
      for (int u = 0; u < kStreamChunkVec; ++u) {
        const int v = (chunk * kStreamChunkVec + u) * NT + tid;
        const u32 ks[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool c = (ks[j] >> 21) >= prefix;
          const u64 m = __ballot(c);
          if (c) {
            const int pos = (int)__builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, (u32)at));
            if (pos < gcap)  // (the histogram promises that it fits)
              __hip_atomic_store(&gl[pos], ((u64)ks[j] << 32) | (u32)(4 * v + j), __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_AGENT);
          }
          at += __popcll(m);
        }
      }
    }
    // The entries travel as device-scope atomic stores and loads (they pass the L2 of the XCD they were written
    // on), and every store of this workgroup has been acknowledged before it counts itself done: no fence, which
    // here would write back and invalidate a whole L2 under the feet of the workgroups still reading keys.  The
    // last workgroup to arrive goes on.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0) s_flag[2] = __hip_atomic_fetch_add(&sy[1], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_flag[2] != n_chunks - 1) return;
    if (tid == 0) {
      sy[0] = 0;
      sy[1] = 0;
    }
    was_valid = A.valid[p] != 0;
    diff_slot_tokens<NT>(A.slot_idx + (size_t)p * k_max, k, pre_tok);
    lds_zero<NT>(s_dyn, 3 * bm_words);
    if (tid < 2) s_flag[tid] = 0;
    my_rounds = (n_list + NT - 1) / NT;
#pragma unroll
    for (int i = 0; i < kMine; ++i) {
      u64 ent = 0ull;
      if (i < my_rounds)
        if (i * NT + tid < n_list) ent = __hip_atomic_load(&gl[i * NT + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ekey[i] = (u32)(ent >> 32);
      eidx[i] = (int)(u32)ent;
    }
    __syncthreads();
    // entries above the bin are in the set for sure
#pragma unroll
    for (int i = 0; i < kMine; ++i)
      if (i < my_rounds)
        if ((ekey[i] >> 21) > prefix) {
          atomicOr(&s_new[eidx[i] >> 5], 1u << (eidx[i] & 31));
          ekey[i] = 0u;
        }
    have_list = true;
  } else {
    if (chunk != 0) return;
    was_valid = A.valid[p] != 0;
    diff_slot_tokens<NT>(A.slot_idx + (size_t)p * k_max, k, pre_tok);
    lds_zero<NT>(s_dyn, 3 * bm_words);
    // f(key, index) for every key of the pair, kBatch vector loads per thread in flight; uniform trip count, all
    // lanes active in f (vectors past the end read as zeros)
    auto stream = [&](auto&& f) {
      for (int v0 = 0; v0 < nvec; v0 += kBatch * NT) {
        v4u kq[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const int v = v0 + u * NT + tid;
          kq[u] = v < nvec ? kp4[v] : v4u{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const int v = v0 + u * NT + tid;
          f(kq[u].x, 4 * v);
          f(kq[u].y, 4 * v + 1);
          f(kq[u].z, 4 * v + 2);
          f(kq[u].w, 4 * v + 3);
        }
      }
    };
    const int part = A.list_cap / NW;  // at most 64 * kMine
    u64* my_ent = l_ent + wave * part;
    int n_mine = 0;  // wave-uniform
    for (;;) {
      if (in_bin <= kStreamLimit && shift > 0) {
        __syncthreads();
        if (tid < 2) s_flag[tid] = 0;
        __syncthreads();
        n_mine = 0;
        stream([&](u32 key, int idx) {
          const u32 top = key >> shift;
          if (top > prefix) atomicOr(&s_new[idx >> 5], 1u << (idx & 31));  // fewer than k keys in all
          const bool c = top == prefix;
          const u64 m = __ballot(c);
          if (c) {
            const int pos = (int)__builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, (u32)n_mine));
            my_ent[min(pos, part - 1)] = ((u64)key << 32) | (u32)idx;
          }
          n_mine += __popcll(m);
        });
        if (n_mine > part - 1 && lane == 0) s_flag[0] = 1;
        __syncthreads();
        if (s_flag[0] == 0) {
          have_list = true;
          break;
        }
      }
      if (shift == 0) break;
      // one radix level down: bits 20..10, then bits 9..0
      const int sub = shift == 21 ? 10 : 0;
      const int nb = shift == 21 ? kBins : 1024;
      __syncthreads();
      lds_zero<NT>(s_hist, nb);
      __syncthreads();
      stream([&](u32 key, int) {
        if ((key >> shift) == prefix) atomicAdd(&s_hist[(key >> sub) & (u32)(nb - 1)], 1u);
      });
      __syncthreads();
      const u32 b = (u32)find_bin<NT, 1>(s_hist, nb, need, &above, s_wave, s_res, nullptr, &in_bin);
      need -= above;
      prefix = (prefix << (shift - sub)) | b;
      shift = sub;
    }
    if (have_list) {
      my_rounds = (n_mine + 63) >> 6;
#pragma unroll
      for (int i = 0; i < kMine; ++i) {
        u64 ent = 0ull;
        if (i < my_rounds)
          if (i * 64 + lane < n_mine) ent = my_ent[i * 64 + lane];
        ekey[i] = (u32)(ent >> 32);
        eidx[i] = (int)(u32)ent;
      }
    } else {
      // T = prefix is known exactly; `need` of the keys equal to it belong to the set
      const u32 T = prefix;
      stream([&](u32 key, int idx) {
        if (key > T)
          atomicOr(&s_new[idx >> 5], 1u << (idx & 31));
        else if (key == T)
          atomicOr(&s_eq[idx >> 5], 1u << (idx & 31));
      });
    }
  }

  bool all_ties = false;  // uniform: every key equal to T belongs to the set and is already in s_new
  if (have_list) {
    // The entries share the bits above `shift`; T is pinned by the bits below.  First the top 12 of them (all of
    // them if there are no more) in kCandBins bins.
    const u32 lo = prefix << shift;
    const int cshift = shift > 12 ? shift - 12 : 0;
    __syncthreads();
    lds_zero<NT>(s_hist, kCandBins);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kMine; ++i)
      if (i < my_rounds)
        if (ekey[i] != 0u) atomicAdd(&s_hist[(ekey[i] - lo) >> cshift], 1u);
    __syncthreads();
    const u32 b1 = (u32)find_bin<NT, 1>(s_hist, kCandBins, need, &above, s_wave, s_res, nullptr, &in_bin);
    need -= above;
    const u32 lo1 = lo + (b1 << cshift);  // T lies in [lo1, lo1 + 2^cshift)
    if (cshift == 0) {
      prefix = lo1;
      all_ties = need == in_bin;
    } else if (in_bin <= 64) {
      // the few keys of that bin are gathered and every wave ranks them by itself
#pragma unroll
      for (int i = 0; i < kMine; ++i)
        if (i < my_rounds)
          if (ekey[i] - lo1 < (1u << cshift)) s_small[atomicAdd(&s_flag[1], 1)] = ekey[i];
      __syncthreads();
      const int n_small = __builtin_amdgcn_readfirstlane(in_bin);
      const u32 v = lane < n_small ? s_small[lane] : 0u;
      int gt = 0, eq = 0;  // keys of the bin above / equal to this lane's (itself included)
      for (int j = 0; j < n_small; ++j) {
        const u32 x = (u32)__builtin_amdgcn_readlane((int)v, j);
        gt += (int)(x > v);
        eq += (int)(x == v);
      }
      const u64 holds = __ballot(lane < n_small && gt < need && need <= gt + eq);
      const int from = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)holds) - 1);
      prefix = (u32)__builtin_amdgcn_readlane((int)v, from);
      need -= __builtin_amdgcn_readlane(gt, from);
      all_ties = need == __builtin_amdgcn_readlane(eq, from);
    } else {
      // one more level over the list: the cshift (at most 9) bits left, in 1024 bins
      lds_zero<NT>(s_hist, 1024);
      __syncthreads();
#pragma unroll
      for (int i = 0; i < kMine; ++i)
        if (i < my_rounds)
          if (ekey[i] - lo1 < (1u << cshift)) atomicAdd(&s_hist[ekey[i] - lo1], 1u);
      __syncthreads();
      const u32 b2 = (u32)find_bin<NT, 1>(s_hist, 1024, need, &above, s_wave, s_res, nullptr, &in_bin);
      need -= above;
      prefix = lo1 + b2;
      all_ties = need == in_bin;
    }
    const u32 T = prefix;  // > 0: the empty entries (key 0) fall through
#pragma unroll
    for (int i = 0; i < kMine; ++i) {
      if (i < my_rounds) {
        if (ekey[i] > T || (all_ties && ekey[i] == T))
          atomicOr(&s_new[eidx[i] >> 5], 1u << (eidx[i] & 31));
        else if (ekey[i] == T)
          atomicOr(&s_eq[eidx[i] >> 5], 1u << (eidx[i] & 31));
      }
    }
  }
  if (tid == 0 && have_list) atomicAdd(&A.stats[6], 1ull);
  __syncthreads();
  // kStreamMaxN keys = 4096 bitmap words.  The candidate list is dead by now: its room stages the diff's lists if
  // they fit.
#define QSAC_DIFF_ARGS                                                                                              \
  s_new, s_eq, s_old, was_valid, need, words, k, A.slot_idx + (size_t)p * k_max,                                    \
      A.set_sorted + (size_t)p * k_max, A.topk_idx + (size_t)p * k, A.hit_mask + (size_t)p * k,                      \
      A.miss_slot + (size_t)p * k_max, A.miss_tok + (size_t)p * k_max, A.fetch_tok + (size_t)p * k_max,              \
      A.miss_count + p, A.valid + p, A.stats, src.slot[p % A.Hkv] >= 0, src.host_row_bytes, s_wave
  if (3 * k + (k + 3) / 4 <= 2 * A.list_cap) {
    int* const room = reinterpret_cast<int*>(l_ent);
    DiffStage st;
    st.ms = room;
    st.mt = room + k;
    st.tk = room + 2 * k;
    st.hm = reinterpret_cast<uint8_t*>(room + 3 * k);
    diff_phases<NT, kStreamMaxN / 32 / NT, true>(QSAC_DIFF_ARGS, st, all_ties, pre_tok);
  } else {
    diff_phases<NT, kStreamMaxN / 32 / NT, false>(QSAC_DIFF_ARGS, DiffStage(), all_ties, pre_tok);
  }
#undef QSAC_DIFF_ARGS
}

// ---------------------------------------------------------------- fill

// Copies the rows named by a pair's miss list into its slots.  A 16-lane group moves one
// 256-byte row with one 16-byte load per lane; each group has four K and four V loads in
// flight before the first store, which is what keeps enough reads outstanding when the
// source is host memory behind PCIe.
__global__ __launch_bounds__(256) void qsac_fill_kernel(const int* __restrict__ miss_count,
                                                        const int* __restrict__ miss_slot,
                                                        const int* __restrict__ miss_tok,
                                                        FillSrc src, v4u* __restrict__ K_slots,
                                                        v4u* __restrict__ V_slots, int Hkv, int64_t N,
                                                        int k_max) {
  const int p = blockIdx.y;
  const int m = miss_count[p];
  const int e0 = blockIdx.x * kFillRows;
  if (e0 >= m) return;
  const int c = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int* ms = miss_slot + (size_t)p * k_max;
  const int* mt = miss_tok + (size_t)p * k_max;
  const v4u *Ks, *Vs;
  fill_rows_of(src, p, Hkv, N, Ks, Vs);
  v4u* Kd = K_slots + (size_t)p * k_max * kRowU4;
  v4u* Vd = V_slots + (size_t)p * k_max * kRowU4;
  int slot[4];
  v4u kr[4], vr[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int e = e0 + u * 16 + grp;
    slot[u] = -1;
    if (e < m) {
      slot[u] = ms[e];
      const size_t tok = (size_t)mt[e];
      kr[u] = Ks[tok * kRowU4 + c];
      vr[u] = Vs[tok * kRowU4 + c];
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (slot[u] >= 0) {
      Kd[(size_t)slot[u] * kRowU4 + c] = kr[u];
      Vd[(size_t)slot[u] * kRowU4 + c] = vr[u];
    }
}

// The same copy for the staggered schedule, where it runs on the second stream beside the scoring of the next
// batch slice: a small, fixed number of workgroups (the grid) walks the miss lists of all P pairs of a slice laid
// end to end, a 16-lane group per row, two rows of K and V (four 16-byte loads) in flight per lane.  That is all a PCIe link
// needs to stay full (measured: 16 workgroups with two loads per lane in flight read pinned memory at 57 GB/s), and
// it matters that it is no more: host reads wait microseconds in the queues they share with everybody's HBM reads,
// and a kernel that keeps tens of MiB of them in flight slows an HBM stream beside it tenfold and more (a 512-MiB
// read: 79 us alone, 110 us beside 16 such workgroups, 4.2 ms beside 2048 with eight loads per lane).
__global__ __launch_bounds__(256) void qsac_fill_trickle_kernel(const int* __restrict__ miss_count,
                                                                const int* __restrict__ miss_slot,
                                                                const int* __restrict__ miss_tok, FillSrc src,
                                                                v4u* __restrict__ K_slots, v4u* __restrict__ V_slots,
                                                                int Hkv, int64_t N, int k_max, int P) {
  // The miss lists of the P pairs laid end to end: s_pre[p] rows come before pair p's.  Every workgroup builds the
  // same table (P ints of dynamic LDS, plus one) and takes every gridDim.x-th run of 32 rows.
  extern __shared__ int s_pre[];
  for (int p = threadIdx.x; p < P; p += 256) s_pre[p + 1] = miss_count[p];
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    s_pre[0] = 0;
    for (int p = 1; p <= P; ++p) {
      run += s_pre[p];
      s_pre[p] = run;
    }
  }
  __syncthreads();
  const int R = s_pre[P];
  const int c = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int stride = (int)gridDim.x * 32;
  int pp[2] = {0, 0};  // the pair a row belongs to only ever moves forward
  // entry of row r (pair, slot, token); the list entries of the next round are requested while this round's rows
  // are on their way, so that a round costs one trip over the link, not a trip to the lists and then one
  struct Entry {
    int p, slot, tok;
  };
  auto entry = [&](int r, int u) {
    Entry en = {0, -1, 0};
    if (r < R) {
      int p = pp[u];
      while (r >= s_pre[p + 1]) ++p;
      pp[u] = p;
      const int e = r - s_pre[p];
      en.p = p;
      en.slot = miss_slot[(size_t)p * k_max + e];
      en.tok = miss_tok[(size_t)p * k_max + e];
    }
    return en;
  };
  int r0 = (int)blockIdx.x * 32 + grp;
  Entry nxt[2] = {entry(r0, 0), entry(r0 + 16, 1)};
  for (; r0 < R; r0 += stride) {
    const Entry cur[2] = {nxt[0], nxt[1]};
    v4u kr[2], vr[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
      if (cur[u].slot >= 0) {
        const v4u *Ks, *Vs;
        fill_rows_of(src, cur[u].p, Hkv, N, Ks, Vs);
        kr[u] = Ks[(size_t)cur[u].tok * kRowU4 + c];
        vr[u] = Vs[(size_t)cur[u].tok * kRowU4 + c];
      }
    nxt[0] = entry(r0 + stride, 0);
    nxt[1] = entry(r0 + stride + 16, 1);
#pragma unroll
    for (int u = 0; u < 2; ++u)
      if (cur[u].slot >= 0) {
        K_slots[((size_t)cur[u].p * k_max + cur[u].slot) * kRowU4 + c] = kr[u];
        V_slots[((size_t)cur[u].p * k_max + cur[u].slot) * kRowU4 + c] = vr[u];
      }
  }
}

// ---------------------------------------------------------------- push-mode transfer

// Push mode (Section 5.2 of the paper, GPU-centric synchronization; Section 6.2, zero-copy transfer engine): the
// GPU hands the compacted miss lists to host transfer threads through a mailbox in pinned host memory and a
// request flag (the paper's Flag1); the threads copy the rows into the cache slots and answer with a completion
// flag (Flag2), which a polling kernel waits for.  Mailbox layout (32-bit words): flag1 at word 0, flag2 at word
// 16, the count of polls that gave up at word 32 (each on a cache line of its own), then count[P], slot[P][k_max],
// tok[P][k_max] from word kPushHeaderWords on.
constexpr int kPushFlag1 = 0, kPushFlag2 = 16, kPushTimeouts = 32, kPushHeaderWords = 64;

// One workgroup per pair copies the pair's miss list into the mailbox.  The last workgroup to finish takes the
// next sequence number and publishes it as Flag1.  state: [0] sequence number of the last request, [1] workgroups
// done in this launch, [2] polls that gave up.
__global__ __launch_bounds__(256) void qsac_publish_kernel(const int* __restrict__ miss_count,
                                                           const int* __restrict__ miss_slot,
                                                           const int* __restrict__ miss_tok, u32* __restrict__ box,
                                                           u32* __restrict__ state, int k_max, int P) {
  const int p = blockIdx.x;
  const int m = miss_count[p];
  int* h_count = reinterpret_cast<int*>(box + kPushHeaderWords);
  int* h_slot = h_count + P + (size_t)p * k_max;
  int* h_tok = h_count + P + (size_t)P * k_max + (size_t)p * k_max;
  const int* ms = miss_slot + (size_t)p * k_max;
  const int* mt = miss_tok + (size_t)p * k_max;
  for (int i = threadIdx.x; i < m; i += 256) {
    h_slot[i] = ms[i];
    h_tok[i] = mt[i];
  }
  if (threadIdx.x == 0) h_count[p] = m;
  // Every workgroup releases its own stores to the host before it counts itself done: workgroups run on
  // different XCDs, host memory is cached in each XCD's L2, and the release that goes with Flag1 below writes
  // back only the L2 of the one workgroup that executes it.
  __threadfence_system();
  __syncthreads();
  if (threadIdx.x == 0) {
    const u32 done = __hip_atomic_fetch_add(&state[1], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (done == (u32)P - 1) {
      state[1] = 0;
      const u32 seq = state[0] + 1;
      state[0] = seq;
      __hip_atomic_store(box + kPushFlag1, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
  }
}

// Waits until the host has answered the last request (Flag2 has reached its sequence number), for at most
// budget_ticks of the constant 100-MHz clock.  Giving up is recorded in state[2] and in the mailbox; either way
// the kernel ends, so the stream never hangs on a host that does not answer.
__global__ __launch_bounds__(64) void qsac_poll_kernel(u32* __restrict__ box, u32* __restrict__ state,
                                                       unsigned long long budget_ticks) {
  if (threadIdx.x != 0) return;
  const u32 want = state[0];
  const unsigned long long t0 = wall_clock64();
  bool ok = false;
  for (;;) {
    const u32 f = __hip_atomic_load(box + kPushFlag2, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM);
    if ((int)(f - want) >= 0) {
      ok = true;
      break;
    }
    if (wall_clock64() - t0 > budget_ticks) break;
    __builtin_amdgcn_s_sleep(16);
  }
  if (!ok) {
    const u32 n = state[2] + 1;
    state[2] = n;
    __hip_atomic_store(box + kPushTimeouts, n, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

// ---------------------------------------------------------------- attention

// which: 0 = every pair, 1 = pairs that reused, 2 = pairs that missed.
__device__ __forceinline__ bool pair_selected(int which, const uint8_t* reuse_flags, int p) {
  return which == 0 || (which == 1) == (reuse_flags[p] != 0);
}

// Workgroup (split, pair): slots [split*rows, split*rows + rows) of the pair, all G query heads; both
// contractions of softmax(q K_c^T / sqrt(d)) V_c (Section 2.1 of the paper) run on the matrix cores.
// Wave w takes the 16-slot tiles w, w+4, ... of the range.  Per tile:
//   - K and V rows arrive by fully coalesced loads (lane l: row 4j + l/16 of the tile, 16-byte piece
//     l%16, j = 0..3) and are parked in two wave-private LDS tiles;
//   - logits, transposed: S^T = K Q^T with the K tile as the A operand (row = slot) and the zero-padded
//     query group as the B operand (column = query), four v_mfma_f32_16x16x32.  Lane l then holds, for
//     query l%16, the logits of slots 4*(l/16) .. +3: exactly where the B operand of the second product
//     wants that query's weights, so the weights never move between lanes;
//   - online softmax per lane (its query; tile maximum over the four lanes that share the query);
//   - O^T += V^T P, eight v_mfma_f32_16x16x32, one per block of 16 channels: the A operand (row =
//     channel, contraction over slots) comes out of the V tile through the transposing LDS load
//     (ds_read_b64_tr_b16); the B operand holds each weight twice, as hi + lo 16-bit parts (the
//     contraction index runs over 16 slots x {hi, lo}), which keeps 16 significant bits of every
//     weight: a weight rounded to one bfloat16 would cost up to 0.4 % of a dominant V row.
// acc[blk][r] of lane l is channel 16 blk + 4 (l/16) + r of query l%16; lanes with l%16 >= G carry
// zero padding.  Waves are merged through LDS; the split's (max, sum, unnormalised output) goes to
// the workspace for qsac_combine_kernel, or, when the pair has a single split, the output is written
// directly.
//
// The next tile's loads are in flight while the current one is consumed.
//
// FETCH ("fill on read"): a slot whose entry in fetch_tok is a token (>= 0) has no row yet: its
// K and V rows are read from the fill sources instead of the slot and written into the slot on
// the way, so the miss fill costs no pass of its own.  Each slot belongs to exactly one lane
// of one workgroup per 16-byte piece, so nothing else reads or writes it during the launch.
typedef __attribute__((ext_vector_type(4))) short s4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t v2u;

struct AttnArgs {
  const uint16_t* q;
  v4u* K_slots;
  v4u* V_slots;
  const int* fetch_tok;
  const int* miss_count;
  const uint8_t* reuse_flags;
  float* part_ml;
  float* part_acc;
  float* out;
  const v4u* K_app;
  const v4u* V_app;
  const DevParams* dp;  // nullptr, or where the number of valid append-buffer rows is read from (then n_app bounds it)
  int64_t N;
  int n_app, app_cap, Hq, Hkv, k, k_max, rows, n_splits, max_splits, which;
};

// LDS of one attention workgroup of NW waves
template <int G, int NW>
struct AttnLds {
  alignas(16) unsigned char ktile[NW][16 * kTilePitch];
  alignas(16) unsigned char vtile[NW][16 * kTilePitch];
  float ml[NW][G][2];
  float acc[NW][G][kD];
};

// 16 slots x 16 channels of an LDS tile as the A operand of a product whose rows are channels and whose
// contraction runs over slots: lane (i = l%16, g = l/16) receives channel c0 + i of slots 4g .. 4g+3.
// The transposing load hands lane 16g + i element i%4 of the 8-byte chunks addressed by lanes
// 16g + i/4 + 4r (r = 0..3) of its group; so lane 16g + s addresses slot 4g + s/4, channels
// c0 + 4(s%4) .. +3.
__device__ __forceinline__ v2u lds_read_tr16(const unsigned char* tile, int c0, int lane) {
  const int g = lane >> 4, s = lane & 15;
  const unsigned char* ptr = tile + (4 * g + (s >> 2)) * kTilePitch + (c0 + 4 * (s & 3)) * 2;
  const s4_t r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4_t __attribute__((address_space(3)))*)ptr);
  return __builtin_bit_cast(v2u, r);
}

// A softmax weight p in [0, 1] as two 16-bit floats of the tile's type with hi + lo = p to 16 (bfloat16) or 22
// (binary16) significant bits.
template <int DT>
__device__ __forceinline__ void split16(float p, u32& hi, u32& lo) {
  if (DT == 0) {
    const _Float16 h = (_Float16)p;
    const _Float16 l = (_Float16)(p - (float)h);
    hi = __builtin_bit_cast(uint16_t, h);
    lo = __builtin_bit_cast(uint16_t, l);
  } else {
    const u32 u = fbits(p);
    hi = u >> 16;  // truncated: the remainder is non-negative and exact in fp32
    const float rem = p - bitsf(u & 0xffff0000u);
    lo = (fbits(rem) + 0x8000u) >> 16;  // rounded to nearest
  }
}

// The work of one attention workgroup of NW waves (all of its threads call this).
template <int DT, int G, bool FETCH, int NW>
__device__ __forceinline__ void attn_body(const AttnArgs& A, const FillSrc& src, int p, int split,
                                          AttnLds<G, NW>& S) {
  constexpr int kStep = NW * 16;  // slots between two tiles of a wave
  v4u* __restrict__ K_slots = A.K_slots;
  v4u* __restrict__ V_slots = A.V_slots;
  float* __restrict__ part_ml = A.part_ml;
  float* __restrict__ part_acc = A.part_acc;
  const int64_t N = A.N;
  // a replayed step reads the row count of the append-only buffer from device memory; the launch is sized for
  // A.n_app rows, and the splits past the valid rows contribute empty partials
  const int n_app = A.dp ? max(0, min(A.dp->n_app, A.n_app)) : A.n_app;
  const int app_cap = A.app_cap, Hq = A.Hq, Hkv = A.Hkv, k = A.k, k_max = A.k_max, rows = A.rows,
            n_splits = A.n_splits, max_splits = A.max_splits;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = lane & 15, quarter = lane >> 4;
  const int b = p / Hkv, h = p % Hkv;
  const v4u* qg = reinterpret_cast<const v4u*>(A.q + ((size_t)b * Hq + (size_t)h * G) * kD);
  v4u qa[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) qa[j] = (m < G) ? qg[m * kRowU4 + quarter * 4 + j] : v4u{0, 0, 0, 0};
  v4u* Kp = K_slots + (size_t)p * k_max * kRowU4;
  v4u* Vp = V_slots + (size_t)p * k_max * kRowU4;
  const v4u *Ks, *Vs;
  fill_rows_of(src, p, Hkv, N, Ks, Vs);
  const int* ft = A.fetch_tok + (size_t)p * k_max;
  const bool fetch = FETCH && A.miss_count[p] > 0;  // uniform over the workgroup
  // Rows k .. k + n_app - 1 of the attended set are the valid rows of the append-only buffer (KV of
  // the tokens generated during decoding, Sections 6.1 and 6.2 of the paper), read in place.
  const v4u* Ka = A.K_app + (size_t)p * app_cap * kRowU4;
  const v4u* Va = A.V_app + (size_t)p * app_cap * kRowU4;

  const float kScale = 1.4426950408889634f * 0.08838834764831845f;  // log2(e) / sqrt(128)
  const float kNegInf = -__builtin_inff();
  // this lane: query m, slots 4*quarter .. +3 of every tile
  float mrun = kNegInf, lrun = 0.f;  // running maximum (log2 domain), this lane's share of the sum
  f4_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = f4_t{0.f, 0.f, 0.f, 0.f};

  const int s_begin = split * rows;
  const int s_end = min(s_begin + rows, k + n_app);
  const int tw = s_begin + wave * 16;  // uniform over the wave: every lane takes part in the MFMAs

  // tokens to fetch for this lane's four rows of the tile at t0 (-1: the row is in its slot).
  // Rows past the end of the range repeat the last row, so that what is loaded is always real data.
  auto load_tok = [&](int t0, int (&tok)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int row = t0 + 4 * j + quarter;
      row = row < s_end ? row : s_end - 1;
      tok[j] = (fetch && row < k) ? ft[row] : -1;
    }
  };
  // issue the loads of this lane's four K (or V) rows of the tile at t0.  Slot rows are streamed (read once per
  // step); rows that come from the fill source keep plain loads: they often still sit in the last-level cache
  // after the scoring pass.
  auto load_tile = [&](int t0, const int (&tok)[4], v4u (&dst)[4], const v4u* slots, const v4u* from_src,
                       const v4u* app) {
    if (FETCH && fetch) {  // uniform: a pair that reused never looks at tokens
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int row = t0 + 4 * j + quarter;
        row = row < s_end ? row : s_end - 1;
        const v4u* from = row < k ? slots + (size_t)row * kRowU4 : app + (size_t)(row - k) * kRowU4;
        if (tok[j] >= 0)
          dst[j] = from_src[(size_t)tok[j] * kRowU4 + m];
        else
          dst[j] = __builtin_nontemporal_load(from + m);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int row = t0 + 4 * j + quarter;
        row = row < s_end ? row : s_end - 1;
        const v4u* from = row < k ? slots + (size_t)row * kRowU4 : app + (size_t)(row - k) * kRowU4;
        dst[j] = __builtin_nontemporal_load(from + m);
      }
    }
  };
  // fetched rows go into their slots; the tile goes into LDS
  auto stage = [&](int t0, const int (&tok)[4], const v4u (&val)[4], v4u* slots, unsigned char* tile) {
    if (FETCH && fetch) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int row = t0 + 4 * j + quarter;
        if (tok[j] >= 0 && row < s_end) slots[(size_t)row * kRowU4 + m] = val[j];
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) *reinterpret_cast<v4u*>(tile + (4 * j + quarter) * kTilePitch + m * 16) = val[j];
    __builtin_amdgcn_wave_barrier();
  };
  unsigned char* ktile = S.ktile[wave];
  unsigned char* vtile = S.vtile[wave];
  v4u pb;    // this tile's weights as the B operand of the second product
  float al;  // this tile's rescale factor of what has been accumulated so far
  // K tile in LDS -> logits -> online softmax
  auto softmax_tile = [&](int t0) {
    f4_t sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const v4u kb = *reinterpret_cast<const v4u*>(ktile + m * kTilePitch + (quarter * 4 + j) * 16);
      sc = mfma16<DT>(kb, qa[j], sc);
    }
    // sc[r]: logit of slot t0 + 4*quarter + r for query m
    float sv[4];
    float tmax = kNegInf;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      sv[r] = (t0 + 4 * quarter + r < s_end) ? sc[r] * kScale : kNegInf;
      tmax = fmaxf(tmax, sv[r]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));  // finite: slot t0 is real
    const float mnew = fmaxf(mrun, tmax);
    al = (mrun == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(mrun - mnew);
    u32 hi[4], lo[4];
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float pw = (sv[r] == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(sv[r] - mnew);
      psum += pw;
      split16<DT>(pw, hi[r], lo[r]);
    }
    lrun = lrun * al + psum;
    mrun = mnew;
    pb = v4u{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
  };
  // V tile in LDS -> O^T <- O^T * alpha + V^T [P_hi ; P_lo]
  auto fold_v = [&]() {
#pragma unroll
    for (int blk = 0; blk < 8; ++blk) {
      const v2u vt = lds_read_tr16(vtile, 16 * blk, lane);
      const v4u va = {vt.x, vt.y, vt.x, vt.y};  // V^T against the hi parts, then against the lo parts
      f4_t c = acc[blk];
#pragma unroll
      for (int r = 0; r < 4; ++r) c[r] *= al;
      acc[blk] = mfma16<DT>(va, pb, c);
    }
    __builtin_amdgcn_wave_barrier();
  };

  {
    // One K and one V register set: the next tile's K loads are issued as soon as this tile's K sits in LDS,
    // the next V loads as soon as this tile's V does.  Tokens run one tile further ahead.
    int tokC[4] = {-1, -1, -1, -1}, tokN[4] = {-1, -1, -1, -1};
    v4u kk[4], vv[4];
    int t0 = tw;
    if (t0 < s_end) {
      if (FETCH && fetch) load_tok(t0, tokC);
      load_tile(t0, tokC, kk, Kp, Ks, Ka);
      load_tile(t0, tokC, vv, Vp, Vs, Va);
      if (FETCH && fetch && t0 + kStep < s_end) load_tok(t0 + kStep, tokN);
    }
    for (; t0 < s_end; t0 += kStep) {
      const bool more = t0 + kStep < s_end;
      stage(t0, tokC, kk, Kp, ktile);
      if (more) load_tile(t0 + kStep, tokN, kk, Kp, Ks, Ka);
      softmax_tile(t0);
      stage(t0, tokC, vv, Vp, vtile);
      if (more) {
        load_tile(t0 + kStep, tokN, vv, Vp, Vs, Va);
        if (FETCH && fetch) {
#pragma unroll
          for (int j = 0; j < 4; ++j) tokC[j] = tokN[j];
          if (t0 + 2 * kStep < s_end) load_tok(t0 + 2 * kStep, tokN);
        }
      }
      fold_v();
    }
  }

  // the four lanes of a query hold different slots under the same maximum
  lrun += __shfl_xor(lrun, 16);
  lrun += __shfl_xor(lrun, 32);
  if (m < G) {
    if (quarter == 0) {
      S.ml[wave][m][0] = mrun;
      S.ml[wave][m][1] = lrun;
    }
#pragma unroll
    for (int blk = 0; blk < 8; ++blk) *reinterpret_cast<f4_t*>(&S.acc[wave][m][16 * blk + 4 * quarter]) = acc[blk];
  }
  __syncthreads();
  float* out_p = A.out + ((size_t)b * Hq + (size_t)h * G) * kD;
  for (int i = threadIdx.x; i < G * kD; i += NW * 64) {
    const int g = i >> 7, d = i & 127;
    float M = kNegInf;
#pragma unroll
    for (int w = 0; w < NW; ++w) M = fmaxf(M, S.ml[w][g][0]);
    float L = 0.f, Acc = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float mw = S.ml[w][g][0];
      const float wt = (mw == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(mw - M);
      L += S.ml[w][g][1] * wt;
      Acc += S.acc[w][g][d] * wt;
    }
    if (n_splits == 1) {
      out_p[i] = Acc / L;
    } else {
      const size_t slot = ((size_t)p * G + g) * max_splits + split;
      part_acc[slot * kD + d] = Acc;
      if (d == 0) {
        part_ml[slot * 2 + 0] = M;
        part_ml[slot * 2 + 1] = L;
      }
    }
  }
}

template <int DT, int G, bool FETCH>
__global__ __launch_bounds__(256) void qsac_attn_kernel(AttnArgs A, FillSrc src) {
  const int p = blockIdx.y, split = blockIdx.x;
  if (!pair_selected(A.which, A.reuse_flags, p)) return;
  __shared__ AttnLds<G, 4> S;
  attn_body<DT, G, FETCH, 4>(A, src, p, split, S);
}

// One workgroup per query head: merges the attention splits and normalises.  128 threads (one
// per channel) times blockDim.x / 128 groups (1 or 4); group j takes the splits 8j .. 8j+7,
// 8(j + groups) .. and the groups are merged through LDS.
// (Merging inside the attention kernel, by the last workgroup of a pair to finish, needs a
// device-scope release/acquire per workgroup, which on this multi-die part writes back and
// invalidates L2 and cost ten times what this launch does.)
__global__ __launch_bounds__(512) void qsac_combine_kernel(const float* __restrict__ part_ml,
                                                           const float* __restrict__ part_acc,
                                                           const uint8_t* __restrict__ reuse_flags,
                                                           float* __restrict__ out, int Hq, int Hkv, int G,
                                                           int n_splits, int max_splits, int which) {
  const int pg = blockIdx.x;  // p * G + g
  const int p = pg / G, g = pg % G;
  if (!pair_selected(which, reuse_flags, p)) return;
  __shared__ float s_m[4][kD], s_l[4][kD], s_a[4][kD];
  const int d = threadIdx.x & 127, grp = threadIdx.x >> 7, groups = blockDim.x >> 7;
  const float kNegInf = -__builtin_inff();
  const float* ml = part_ml + (size_t)pg * max_splits * 2;
  const float* pa = part_acc + (size_t)pg * max_splits * kD;
  // eight splits at a time: their loads are all issued before the first is used, and the chunks
  // are merged online
  float M = kNegInf, L = 0.f, A = 0.f;
  for (int s0 = grp * 8; s0 < n_splits; s0 += groups * 8) {
    float mv[8], lv[8], av[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int sp = s0 + i;
      const bool in = sp < n_splits;
      mv[i] = in ? ml[sp * 2] : kNegInf;
      lv[i] = in ? ml[sp * 2 + 1] : 0.f;
      av[i] = in ? pa[(size_t)sp * kD + d] : 0.f;
    }
    float Mc = M;
#pragma unroll
    for (int i = 0; i < 8; ++i) Mc = fmaxf(Mc, mv[i]);
    const float w0 = (M == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(M - Mc);
    L *= w0;
    A *= w0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float wt = (mv[i] == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(mv[i] - Mc);
      L += lv[i] * wt;
      A += av[i] * wt;
    }
    M = Mc;
  }
  if (groups > 1) {  // uniform
    s_m[grp][d] = M;
    s_l[grp][d] = L;
    s_a[grp][d] = A;
    __syncthreads();
    if (grp != 0) return;
    float Mc = M;
    for (int j = 1; j < groups; ++j) Mc = fmaxf(Mc, s_m[j][d]);
    float Ls = 0.f, As = 0.f;
    for (int j = 0; j < groups; ++j) {
      const float mj = s_m[j][d];
      const float wt = (mj == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(mj - Mc);
      Ls += s_l[j][d] * wt;
      As += s_a[j][d] * wt;
    }
    L = Ls;
    A = As;
  }
  const int b = p / Hkv, h = p % Hkv;
  out[((size_t)b * Hq + (size_t)h * G + g) * kD + d] = A / L;
}

// Eq. (2) weights s_j of the query heads, widened to fp64 where the gate reads them.  They travel as a kernel
// argument, so that setting them needs neither a copy nor a staging buffer.
struct ImportanceArg {
  float v[512];  // QSAC_MAX_KV_HEADS * QSAC_MAX_GROUP query heads at most
};
__global__ __launch_bounds__(256) void qsac_set_importance_kernel(double* __restrict__ importance, ImportanceArg w, int n) {
  for (int i = threadIdx.x; i < n; i += 256) importance[i] = (double)w.v[i];
}

// Clears `n` 32-bit words (used instead of a memset node so that the step can be captured in a graph).
__global__ __launch_bounds__(256) void qsac_zero_kernel(u32* __restrict__ ptr, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) ptr[i] = 0;
}

}  // namespace qsac
